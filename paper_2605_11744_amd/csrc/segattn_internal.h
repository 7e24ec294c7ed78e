// Internal declarations shared by the translation units of libsegattn (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <atomic>
#include <mutex>

#include "segattn.h"

namespace segattn {

constexpr int kMaxKvHeads = 128;
// per (sequence, KV head): pool rows, tail rows, open-segment rows, first visible pool row,
// rows of the retrieved prefix (retrieval mode), 3 unused
constexpr int kMetaInts = 8;

enum MetaSlot { META_POOL = 0, META_TAIL = 1, META_FILL = 2, META_LO = 3, META_RET = 4 };

// Geometry of the cache arena, identical on host and device.
//   [ counters : B*Hkv*8 int32 ][ decode workspace ][ K/V rows ][ attention views ]
// K/V rows of (b, h): K block of cap(h) rows, then V block of cap(h) rows, D bf16 each;
// cap(h) = pool_cap for a PAST head, T + S otherwise.
// Retrieval mode (ret_cap > 0): a PAST head attends to [retrieved prefix ; open segment]
// instead of its pool, read from its attention view: K block of ret_cap + S rows, then the V
// block; rows [ret_cap - R, ret_cap) hold the R retrieved rows, rows from ret_cap on mirror the
// open segment (which is appended to the pool as well).
struct CacheGeom {
  unsigned long long meta_off, ws_off, kv_off, view_off;
  unsigned long long part_off;         // split-prefix workspace of the segment-by-segment prefill (0: none)
  int part_max;                        // most parts a PAST head's prefix may be cut into (1: never split)
  unsigned long long rows_per_seq;     // sum of cap(h) over heads
  unsigned long long pool_cap;         // rows per PAST head
  int ret_cap;                         // rows of retrieved prefix a view can hold; 0: no views
  int ws_splits_past, ws_splits_other; // split-K slots per query head (PAST / other heads): one more
                                       // than the chunks of the largest window (slices need not
                                       // start at a window's first row)
  int decode_chunk;                    // keys per split
};

// One split-K partial of the decode path: D accumulator floats, then the reference maximum and the
// row sum, padded so that every slot starts on a 128-byte line and is written by one workgroup in
// whole lines (slots sharing lines, written from different XCDs, cost the split kernel 13 %).
constexpr int kWsTailFloats = 32;
__host__ __device__ inline int ws_slot_floats(int D) { return D + kWsTailFloats; }

// Everything a kernel needs to know about the problem; passed by value as kernel argument.
struct Problem;
__host__ __device__ inline unsigned long long ws_header_bytes(const Problem &p);
struct Problem {
  int B, Hq, Hkv, g, D, S, T;
  float scale;          // multiplies q.k
  float scale_log2e;    // scale * log2(e)
  int out_fp32;         // `out` holds fp32 instead of bf16
  int fp32_math;        // validation mode: fp32 FMA kernels
  int n_past;           // number of PAST heads
  int tune_waves;       // host only: 0, or the forced waves per workgroup of the D = 128 forward kernel (4 / 8)
  int tune_queue;       // host only: item queues -- 0 the library chooses, 1 never, 2 always, 3 always, small grid
  // Per-head tables as 32-bit words: a kernel indexes them with a workgroup-uniform value, and
  // only whole words of the argument block can be fetched with scalar loads (bytes would go
  // through the vector memory path and cost every workgroup a memory round trip each).
  int policy[kMaxKvHeads];
  int order[kMaxKvHeads];         // KV heads, PAST heads first
  int past_before[kMaxKvHeads];   // number of PAST heads with a smaller index
};

// The decode workspace starts with one int per (sequence, KV head): partials written for its window.
__host__ __device__ inline unsigned long long ws_header_bytes(const Problem &p) {
  return ((unsigned long long)p.B * p.Hkv * 4ull + 127ull) / 128ull * 128ull;
}

// Arguments of the prefill kernels.  SEQ mode (cache == nullptr): q/k/v hold n_rows = N tokens
// per sequence and every segment is processed in this launch.  CTX mode: q/k/v hold the
// n_rows = m new rows of the open segment and the prefix comes from the cache arena.
// n / d for 0 <= n < 2^31 and a divisor d >= 1 that is fixed for a launch: the host prepares
// mul = ceil(2^shift / d) with shift = 31 + ceil(log2 d); then floor(n * mul / 2^shift) is exact
// (n * (mul * d - 2^shift) < 2^31 * 2^ceil(log2 d) = 2^shift) and mul fits 32 bits.  A scalar
// multiply-high and a shift in place of the instruction sequence of an integer division.
struct FastDiv {
  unsigned mul, shift, d;
};
inline FastDiv fast_div_by(long long d) {
  FastDiv f{0u, 0u, 0u};
  if (d < 1 || d >= (1ll << 31)) return f;  // d == 0 marks an unusable entry
  unsigned s = 0;
  while ((1ull << s) < (unsigned long long)d) ++s;
  const unsigned shift = 31 + s;
  const unsigned long long mul = ((1ull << shift) + (unsigned long long)d - 1) / (unsigned long long)d;
  f.mul = (unsigned)mul;
  f.shift = shift;
  f.d = (unsigned)d;
  return f;
}
__host__ __device__ inline int fast_div(int n, const FastDiv &f) {
  return (int)(((unsigned long long)(unsigned)n * f.mul) >> f.shift);
}
__host__ __device__ inline int fast_mod(int n, const FastDiv &f) { return n - fast_div(n, f) * (int)f.d; }
// The divisors of resolve() (segattn_work.h), prepared by the launcher; `ok` == 0: resolve()
// divides as written.
struct ResolveDivs {
  int ok;
  FastDiv per, parts, nqb, nhs, n_first, n_other, batch, per_sub, sub, groups;
};

struct PrefillArgs {
  const unsigned short *q, *k, *v;
  void *out;
  float *lse;
  unsigned char *cache;  // arena base or nullptr
  CacheGeom geom;
  int n_rows;            // N (SEQ; the longest sequence of a packed batch) or m (CTX)
  const int *cu_seqlens; // SEQ mode, packed ragged batch: device [B+1] row offsets, else nullptr
  long long total_rows;  // rows of the packed batch (lse is [Hq, total_rows] then)
  int n_seg;             // segments covered by the launch (1 in CTX mode)
  int q_blocks_per_seg;  // ceil(min(S, n_rows) / rows per workgroup); set by the launcher
  int pair_stride;       // spreads the (segment, sequence, head) groups of non-PAST heads over the XCDs (0 = 1)
  int sub_groups;        // a group's query blocks are dealt into this many interleaved sub-groups (0 = 1) so that
                         // every XCD's share of the non-PAST list is a whole number of (sub-)groups
  // CTX mode, split prefix: the prefix of every PAST head is cut into `parts` pieces, each handled
  // by a workgroup of its own (the last one also takes the open segment); the pieces' normalised
  // fp32 outputs and their LSEs go to the workspace and prefill_part_combine_kernel merges them.
  int parts;             // 0 or 1: no split
  long long min_past_prefix;  // host: fewest prefix rows among the PAST windows (sets how far to split)
  float *part_out;       // [B][parts][n_rows][n_past*g][D]
  float *part_lse;       // [B][parts][n_past*g][n_rows]
  // Work items of the launch (0: the grid size) and, where the workgroups take their items from
  // queues, the counters: next item of XCD y's queue at queue[kQueueStride * y], zero at the start.
  int grid_items;
  unsigned *queue;       // device; nullptr: workgroup i runs item i
  // SEQ mode, retrieved prefixes (stateless retrieval mode): a PAST head attends to [R gathered rows ;
  // own segment]; the rows of (b, segment, PAST head) are R dense rows of D at
  // ret_k / ret_v + (((b * n_seg + segment) * n_past + past index) * R) * D.  nullptr: whole history.
  const unsigned short *ret_k, *ret_v;
  int ret_R;
  ResolveDivs dv;
};
// Fills a.dv for a launch whose fields resolve() reads are final (q_blocks_per_seg, n_seg, parts,
// sub_groups, pair_stride, grid_items); heads_per_wg as passed to resolve().
inline void prepare_resolve_divs(const Problem &p, PrefillArgs &a, int heads_per_wg, long long grid) {
  ResolveDivs &dv = a.dv;
  dv.ok = 0;
  const int nhs = p.g / heads_per_wg;
  const int nqb = a.q_blocks_per_seg;
  const int n_first = ((a.cache != nullptr && a.geom.ret_cap > 0) || a.ret_k != nullptr) ? 0 : p.n_past;
  const int n_other = p.Hkv - n_first;
  const int parts = (a.cache != nullptr && a.parts > 1) ? a.parts : 1;
  const long long past_items = (long long)p.B * n_first * nhs * a.n_seg * nqb * parts;
  const long long items = grid - past_items;
  const int d = a.sub_groups > 1 ? a.sub_groups : 1;
  if (nqb < 1 || nhs < 1 || grid >= (1ll << 31) || nqb % d != 0) return;
  const long long groups = items / nqb;
  const long long stride = a.pair_stride > 0 ? a.pair_stride : 1;
  if (groups > 0 && (groups - 1) * stride >= (1ll << 31)) return;  // the shuffled group index must fit
  dv.per = fast_div_by((long long)p.B * (n_first > 0 ? n_first : 1) * nhs * parts);
  dv.parts = fast_div_by(parts);
  dv.nqb = fast_div_by(nqb);
  dv.nhs = fast_div_by(nhs);
  dv.n_first = fast_div_by(n_first > 0 ? n_first : 1);
  dv.n_other = fast_div_by(n_other > 0 ? n_other : 1);
  dv.batch = fast_div_by(p.B);
  dv.per_sub = fast_div_by(nqb / d);
  dv.sub = fast_div_by(d);
  dv.groups = fast_div_by(groups > 0 ? groups : 1);
  const FastDiv *all[] = {&dv.per, &dv.parts, &dv.nqb, &dv.nhs, &dv.n_first, &dv.n_other, &dv.batch, &dv.per_sub, &dv.sub, &dv.groups};
  for (const FastDiv *f : all)
    if (f->d == 0) return;
  dv.ok = 1;
}
constexpr int kQueueStride = 32;  // unsigned words between two queue counters (128 bytes)
// Host side of the item queues (segattn_prefill_mfma.hip): the counters of this (device, stream),
// or nullptr where the launch has to run one workgroup per item (stream under capture, no set
// left); and the kernel that clears them, to be launched in front of every queued launch.
// The reset and the launch that uses the counters must enter the stream back to back: hold
// item_queue_launch_mutex() around the pair (two host threads may launch into one stream).
unsigned *item_queue_for(hipStream_t st);
hipError_t item_queue_reset(unsigned *queue, hipStream_t st);
std::mutex &item_queue_launch_mutex();
// Grid of a launch of `items` work items whose kernel fits `resident` workgroups on the chip at
// once, under Problem::tune_queue: `items` (one workgroup per item, no queues), or fewer
// workgroups that take their items from the queues.  The library's own choice is the resident
// grid whenever a workgroup would get more than two items (with fewer there is little to balance
// and the counters' reset kernel and first round trip are not earned back).
inline long long item_queue_grid(const Problem &p, long long items, long long resident) {
  if (resident <= 0 || p.tune_queue == 1) return items;
  if (p.tune_queue >= 2 ? items <= 1 : items <= 2 * resident) return items;
  long long launch = resident < items ? resident : items;
  if (p.tune_queue == 3 && items / 3 < launch) launch = items / 3 > 0 ? items / 3 : 1;
  return launch;
}

// Workgroups of one kernel that the device holds at once: asked from the runtime by the first
// launch and kept.  Safe from any number of host threads: racing first calls ask the same
// question and store the same answer.  0: the query failed (asked again by the next launch).
class ResidentCount {
 public:
  int get(const void *kernel, int threads, size_t dynamic_lds) {
    int v = n_.load(std::memory_order_acquire);
    if (v > 0) return v;
    int dev = 0, cus = 0, per_cu = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
        hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, threads, dynamic_lds) != hipSuccess ||
        cus < 1 || per_cu < 1) {
      (void)hipGetLastError();
      return 0;
    }
    v = cus * per_cu;
    n_.store(v, std::memory_order_release);
    return v;
  }

 private:
  std::atomic<int> n_{0};
};

struct DecodeArgs {
  const unsigned short *q, *k_new, *v_new;
  void *out;
  float *lse;
  unsigned char *cache;
  CacheGeom geom;
  long long total_rows;  // visible rows summed over every (sequence, KV head) window
  int rows_per_wg;       // rows per workgroup of the split kernel (>= geom.decode_chunk); set by the launcher
};

struct CopyArgs {
  const unsigned short *k, *v;   // source rows
  unsigned char *cache;
  CacheGeom geom;
  int m;                 // rows per sequence in the source
  int kv_head;           // past_append: target head; otherwise unused
};

// Arguments of the backward kernels (whole-sequence form, positions absolute as in SEQ mode).
struct BwdArgs {
  const unsigned short *q, *k, *v, *dout;  // bf16
  const void *out;                         // forward output: bf16, or fp32 if Problem::out_fp32
  const float *lse;                        // [B,Hq,n]
  float *delta;                            // [B,Hq,n] workspace: sum_d dO*O
  float *nls;                              // [B,Hq,n] workspace: -lse / scale (the dK/dV kernel starts its score
                                           // accumulators there: exp2((q.k - lse/scale) scale log2 e) is the weight)
  void *dq, *dk, *dv;                      // bf16, or fp32 if Problem::out_fp32
  int n;                                   // rows per sequence (packed batch: of the longest sequence)
  const int *cu_seqlens;                   // packed ragged batch: device [B+1] row offsets, else nullptr
  long long total;                         // rows of the packed batch; lse, delta are [Hq,total] then
};

// Where sequence b of a backward call lives: its first row and length in the token-major tensors,
// and the index of (head 0, row 0) and the head stride in lse / delta.
struct SeqSpan {
  long long row0, n, stat0, stat_stride;
};
__device__ inline SeqSpan seq_span(const Problem &p, const BwdArgs &a, int b) {
  SeqSpan s;
  if (a.cu_seqlens) {
    s.row0 = a.cu_seqlens[b];
    s.n = a.cu_seqlens[b + 1] - s.row0;
    s.stat0 = s.row0;
    s.stat_stride = a.total;
  } else {
    s.row0 = (long long)b * a.n;
    s.n = a.n;
    s.stat0 = (long long)b * p.Hq * a.n;
    s.stat_stride = a.n;
  }
  return s;
}
// Sequence of global token row `row` (dense: row / n; packed: binary search in cu_seqlens).
__device__ inline int seq_of_row(const Problem &p, const BwdArgs &a, long long row) {
  if (!a.cu_seqlens) return (int)(row / a.n);
  int lo = 0, hi = p.B - 1;
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (a.cu_seqlens[mid] <= row) lo = mid;
    else hi = mid - 1;
  }
  return lo;
}

// seg_kv_set_lengths: the declared lengths of a chunk of sequences, by value.
constexpr int kLengthsChunk = 128;
struct LengthsArgs {
  int b0, count;                       // sequences b0 .. b0 + count - 1
  int closed[kLengthsChunk], tail[kLengthsChunk], fill[kLengthsChunk];
};

// Gather of the retrieved prefixes of a whole prompt (stateless retrieval mode): for every
// (b, segment >= 1, PAST head) the R rows idx names, from the token-major k / v into dense rows.
struct GatherSeqArgs {
  const unsigned short *k, *v;   // [B, n, Hkv, D]
  const int *idx;                // [B, n_seg, n_past, R] positions (< segment start)
  unsigned short *ret_k, *ret_v; // [B, n_seg, n_past, R, D]
  int n, n_seg, R;
  int rope;                      // re-rotate the gathered K rows to the positions just before their segment
  double inv_freq[64];
};

struct SelectArgs {
  const int *idx;        // [B, n_past, R] pool row numbers
  unsigned char *cache;
  CacheGeom geom;
  int R;
  int rope;              // re-rotate the gathered K rows to the positions just before the segment
  double inv_freq[64];   // theta^(-2i/D), i < D/2
};

// Arguments of the retrieval operator kernels.
struct RetrieveArgs {
  const unsigned short *q_prev;  // [B, m, Hq, D] queries of the previous segment
  unsigned char *cache;
  CacheGeom geom;
  unsigned short *summaries;     // workspace: [B, n_past, nsp, D] bf16
  float *cand_val;               // workspace: [B, n_past, n_chunks, 32]
  int *cand_idx;                 // workspace: same shape
  int *idx_out;                  // [B, n_past, R]
  int m, R, nsp, n_chunks, chunk_rows;
  int n_queries, pool_window, tail_avg, n_anchors, win_before, win_after;
  // Whole-prompt form (k_seq != nullptr; cache unused): the "sequences" the kernels see are the
  // pairs (b, segment i), B * n_seg of them; the pool of (b, i) is rows [0, i S) of k_seq
  // [B, n_rows, Hkv, D] and its query rows are those of segment i - 1 in q_prev [B, n_rows, Hq, D]
  // (m = S).  Segment 0 has an empty pool and gets an unused list.
  const unsigned short *k_seq;
  int n_rows, n_seg;
};

struct RopeArgs {
  unsigned short *q, *k;     // rotated in place
  const long long *pos0;     // device [B]: position of row 0 of every sequence, or nullptr (all 0)
  int rows;
  double inv_freq[64];
};

// ---- helpers usable on host and device ----------------------------------------------------
__host__ __device__ inline unsigned long long head_row_offset(const Problem &p, const CacheGeom &g,
                                                              int h) {
  unsigned long long np = p.past_before[h];
  return np * g.pool_cap + (unsigned long long)(h - (int)np) * (unsigned long long)(p.T + p.S);
}
__host__ __device__ inline unsigned long long head_cap(const Problem &p, const CacheGeom &g, int h) {
  return (p.policy[h] & SEGATTN_PAST) ? g.pool_cap : (unsigned long long)(p.T + p.S);
}
__host__ __device__ inline unsigned long long k_block_off(const Problem &p, const CacheGeom &g, int b,
                                                          int h) {
  return g.kv_off + ((unsigned long long)b * g.rows_per_seq + head_row_offset(p, g, h)) * 2ull *
                        (unsigned long long)p.D * 2ull;
}
__host__ __device__ inline unsigned long long v_block_off(const Problem &p, const CacheGeom &g, int b,
                                                          int h) {
  return k_block_off(p, g, b, h) + head_cap(p, g, h) * (unsigned long long)p.D * 2ull;
}
// Attention view of a PAST head in retrieval mode.
__host__ __device__ inline unsigned long long view_k_off(const Problem &p, const CacheGeom &g, int b, int h) {
  return g.view_off + ((unsigned long long)b * p.n_past + p.past_before[h]) * 2ull *
                          (unsigned long long)(g.ret_cap + p.S) * (unsigned long long)p.D * 2ull;
}
__host__ __device__ inline unsigned long long view_v_off(const Problem &p, const CacheGeom &g, int b, int h) {
  return view_k_off(p, g, b, h) + (unsigned long long)(g.ret_cap + p.S) * (unsigned long long)p.D * 2ull;
}
__host__ __device__ inline bool uses_view(const Problem &p, const CacheGeom &g, int h) {
  return g.ret_cap > 0 && (p.policy[h] & SEGATTN_PAST);
}
// The block the attention kernels read for (b,h): the view in retrieval mode, else the K/V rows.
__host__ __device__ inline unsigned long long attn_k_off(const Problem &p, const CacheGeom &g, int b, int h) {
  return uses_view(p, g, h) ? view_k_off(p, g, b, h) : k_block_off(p, g, b, h);
}
__host__ __device__ inline unsigned long long attn_v_off(const Problem &p, const CacheGeom &g, int b, int h) {
  return uses_view(p, g, h) ? view_v_off(p, g, b, h) : v_block_off(p, g, b, h);
}
// First row of the visible window and first row of the open segment inside the block that
// attn_k_off / attn_v_off name.
__host__ __device__ inline void window_of(const Problem &p, const CacheGeom &g, int h, const int *meta,
                                          int &lo, int &seg_row0) {
  const int pol = p.policy[h];
  if (uses_view(p, g, h)) {
    lo = g.ret_cap - meta[META_RET];
    seg_row0 = g.ret_cap;
  } else if (pol & SEGATTN_PAST) {
    lo = meta[META_LO];
    seg_row0 = meta[META_POOL];
  } else {
    lo = (pol & SEGATTN_TAIL) ? p.T - meta[META_TAIL] : p.T;
    seg_row0 = p.T;
  }
}

// The pool of PAST head kv of "sequence" vb as the retrieval kernels see it.
struct PoolView {
  const unsigned char *k;   // first K row
  long long row_bytes;      // bytes between consecutive rows
  int pool, lo;             // rows held; first visible row
  const unsigned short *q;  // the m previous-segment query rows [m, Hq, D] the summaries are made of
};
__device__ inline PoolView pool_view(const Problem &p, const RetrieveArgs &a, int vb, int kv) {
  PoolView v;
  if (a.k_seq) {
    const int b = vb / a.n_seg, i = vb % a.n_seg;
    v.k = (const unsigned char *)(a.k_seq + ((long long)b * a.n_rows * p.Hkv + kv) * p.D);
    v.row_bytes = (long long)p.Hkv * p.D * 2;
    v.pool = i * p.S;
    v.lo = 0;
    v.q = a.q_prev + ((long long)b * a.n_rows + (long long)(i > 0 ? i - 1 : 0) * p.S) * p.Hq * p.D;
  } else {
    const int *meta = (const int *)(a.cache + a.geom.meta_off) + ((long long)vb * p.Hkv + kv) * kMetaInts;
    v.k = a.cache + k_block_off(p, a.geom, vb, kv);
    v.row_bytes = 2 * p.D;
    v.pool = meta[META_POOL];
    v.lo = meta[META_LO];
    v.q = a.q_prev + (long long)vb * a.m * p.Hq * p.D;
  }
  return v;
}

// ---- decode: counters and split-K workspace (device side) ---------------------------------------
__device__ inline const int *meta_ro(const unsigned char *cache, const CacheGeom &g, const Problem &p, int b,
                                     int h) {
  return (const int *)(cache + g.meta_off) + ((long long)b * p.Hkv + h) * kMetaInts;
}

// The split-K workspace: one int per (b, KV head) window (number of partials written), then the
// partial slots.
__device__ inline int *ws_counts(unsigned char *cache, const CacheGeom &g) { return (int *)(cache + g.ws_off); }
__device__ inline float *ws_slots(unsigned char *cache, const CacheGeom &g, const Problem &p) {
  return (float *)(cache + g.ws_off + ws_header_bytes(p));
}
// split-K slots (ws_slot_floats(D) floats each) before those of (b, query head)
__device__ inline long long ws_slot_base(const Problem &p, const CacheGeom &g, int b, int head) {
  const int kv = head / p.g;
  const long long np = p.past_before[kv];
  const long long per_seq = (long long)p.g * ((long long)p.n_past * g.ws_splits_past +
                                              (long long)(p.Hkv - p.n_past) * g.ws_splits_other);
  const long long before = (long long)p.g * (np * g.ws_splits_past + (kv - np) * g.ws_splits_other);
  const long long mine = (p.policy[kv] & SEGATTN_PAST) ? g.ws_splits_past : g.ws_splits_other;
  return (long long)b * per_seq + before + (long long)(head % p.g) * mine;
}


// ---- launchers (defined in the .hip files) ------------------------------------------------
hipError_t launch_prefill(const Problem &p, const PrefillArgs &a, hipStream_t st);
// bytes of split-prefix workspace for `parts` pieces (fp32 outputs + LSEs of one segment of every sequence)
__host__ __device__ inline unsigned long long part_ws_bytes(const Problem &p, int parts) {
  return (unsigned long long)p.B * parts * p.S * p.n_past * p.g * (unsigned long long)(p.D + 1) * 4ull;
}
hipError_t launch_decode(const Problem &p, const DecodeArgs &a, int B, hipStream_t st);
int decode_mfma_resident(int D);  // workgroups of the matrix-core split kernel the chip holds at once (0: error)
hipError_t launch_decode_split_mfma(const Problem &p, const DecodeArgs &a, long long blocks, hipStream_t st);
hipError_t launch_cache_reset(const Problem &p, unsigned char *cache, const CacheGeom &g, hipStream_t st);
hipError_t launch_cache_append(const Problem &p, const CopyArgs &a, hipStream_t st);
hipError_t launch_cache_commit_seq(const Problem &p, const CopyArgs &a, hipStream_t st);
hipError_t launch_cache_close(const Problem &p, unsigned char *cache, const CacheGeom &g, int add,
                              hipStream_t st);
hipError_t launch_cache_decode_append(const Problem &p, const CopyArgs &a, hipStream_t st);
hipError_t launch_cache_past_append(const Problem &p, const CopyArgs &a, hipStream_t st);
hipError_t launch_cache_evict(const Problem &p, unsigned char *cache, const CacheGeom &g, int kv_head,
                              long long n_oldest, long long keep, hipStream_t st);
hipError_t launch_cache_select(const Problem &p, const SelectArgs &a, hipStream_t st);
hipError_t launch_cache_set_lengths(const Problem &p, unsigned char *cache, const CacheGeom &g, const LengthsArgs &a,
                                    hipStream_t st);
hipError_t launch_retrieve(const Problem &p, const RetrieveArgs &a, hipStream_t st);
hipError_t launch_gather_seq(const Problem &p, const GatherSeqArgs &a, hipStream_t st);
hipError_t launch_rope_apply(const Problem &p, const RopeArgs &a, hipStream_t st);
hipError_t launch_bwd_delta(const Problem &p, const BwdArgs &a, hipStream_t st);
hipError_t launch_bwd_fp32(const Problem &p, const BwdArgs &a, hipStream_t st);
hipError_t launch_bwd_dq(const Problem &p, const BwdArgs &a, hipStream_t st);
hipError_t launch_bwd_mfma(const Problem &p, const BwdArgs &a, hipStream_t st);
int prefill_pair_stride(long long groups);
hipError_t launch_probe(void *buf, long long bytes, int mode, void *sink, hipStream_t st);
constexpr int kClockProbeWaves = 8;  // one per XCD
hipError_t launch_clock_probe(unsigned long long ticks, unsigned long long *out, hipStream_t st);
constexpr int kMfmaProbeFlopsPerWaveIter = 8 * 2 * 32 * 32 * 16;  // eight 32x32x16 products
hipError_t launch_mfma_probe(int iters, int quiet, int workgroups, float *sink, hipStream_t st);

}  // namespace segattn
