// Top-k retrieval operator (Appendix D) for the long-range channel of libsegattn: from the
// previous segment's queries and a long-range head's past pool to the R pool rows that become
// the retrieved prefix.  The paper names the steps but none of their sizes; the sizes are
// parameters here (segattn_retrieval) and the steps are read as follows:
//
//   query construction   last L_q query rows of the previous segment, every query head of the
//                        group: means of consecutive windows of `pool_window` rows, plus the mean
//                        of the last `tail_avg` rows; rounded to bf16 (MFMA operands)
//   scoring              score(row) = max over the summaries of summary . key(row): one pass over
//                        the pool's K rows, HBM-bound (each row read once); the products are a
//                        dense [summaries x 128] x [128 x rows] contraction and run on the
//                        matrix cores so that the scan stays bandwidth-bound
//   top-k / anchors      the n_anchors rows with the highest scores, ties to the lower row.  (For
//                        any k >= n_anchors these are the anchors that "per-summary top-k,
//                        de-duplicate, keep the best" yields.)  Two levels: every chunk of 1024
//                        or 4096 rows (small chunks when few heads have to fill the chip)
//                        keeps its own best n_anchors next to the scores in LDS -- scores never
//                        go to HBM -- and one workgroup per head merges the candidates
//   window expansion     anchors in descending score order add rows a - win_before .. a + win_after
//                        (clipped to the visible pool, ascending, rows already in skipped) until
//                        R rows are in; then the earliest visible rows pad to R; sorted output
#include "segattn_internal.h"

namespace segattn {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

constexpr int kMaxAnchors = 32;

// (value, row) pairs ordered by value descending, then row ascending
__device__ inline bool better(float v, int i, float w, int j) { return v > w || (v == w && i < j); }

// Wave-wide best (value, row); every lane gets the result.  The four exchanges inside a row of 16
// lanes are DPP moves (a register-to-register step of a few cycles each), the exchange between
// rows one LDS-crossbar shuffle, the one between half-waves a lane swap: a third of the latency of
// six crossbar shuffles, and this reduction sits inside loops of n_anchors rounds.
__device__ inline void wave_best(float &v, int &i) {
#define SEGATTN_BEST_STEP(CTRL)                                                                         \
  do {                                                                                                \
    const float w_ = __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(v), CTRL, 0xF, 0xF, true)); \
    const int j_ = __builtin_amdgcn_mov_dpp(i, CTRL, 0xF, 0xF, true);                                   \
    if (better(w_, j_, v, i)) {                                                                       \
      v = w_;                                                                                         \
      i = j_;                                                                                         \
    }                                                                                                 \
  } while (0)
  SEGATTN_BEST_STEP(0xB1);   // quad_perm [1,0,3,2]
  SEGATTN_BEST_STEP(0x4E);   // quad_perm [2,3,0,1]
  SEGATTN_BEST_STEP(0x141);  // row_half_mirror
  SEGATTN_BEST_STEP(0x140);  // row_mirror: all 16 lanes of a row agree
#undef SEGATTN_BEST_STEP
  {
    const float w = __shfl_xor(v, 16);
    const int j = __shfl_xor(i, 16);
    if (better(w, j, v, i)) {
      v = w;
      i = j;
    }
  }
  {  // the two halves: one element of each pair is the lane's own value, the other its partner's
    const auto sv = __builtin_amdgcn_permlane32_swap(__float_as_int(v), __float_as_int(v), false, false);
    const auto si = __builtin_amdgcn_permlane32_swap(i, i, false, false);
    const float v0 = __int_as_float(sv[0]), v1 = __int_as_float(sv[1]);
    const bool second = better(v1, si[1], v0, si[0]);
    v = second ? v1 : v0;
    i = second ? si[1] : si[0];
  }
}

// Workgroup-wide best (value, row); every thread gets the result.  sm: 2 * 4 words of LDS.
__device__ inline void block_best(float &v, int &i, float *sm_v, int *sm_i) {
  wave_best(v, i);
  const int wave = threadIdx.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) {
    sm_v[wave] = v;
    sm_i[wave] = i;
  }
  __syncthreads();
  v = sm_v[0];
  i = sm_i[0];
#pragma unroll
  for (int w = 1; w < 4; ++w)
    if (better(sm_v[w], sm_i[w], v, i)) {
      v = sm_v[w];
      i = sm_i[w];
    }
}

// ---- query summaries: [B, n_past, NSP, D] bf16, NSP = g * n_sum rounded up to 32 (the padding
//      repeats summary 0, which cannot change a maximum).  One workgroup per (b, PAST head).
template <int D>
__global__ __launch_bounds__(256) void retrieve_summaries_kernel(const Problem p, const RetrieveArgs a) {
  constexpr int CH = D / 8;  // a thread forms 8 channels of one summary
  const int b = blockIdx.x / p.n_past, np = blockIdx.x % p.n_past;  // b: sequence, or (sequence, segment)
  const int kv = p.order[np];
  const PoolView pv = pool_view(p, a, b, kv);
  const int L = a.n_queries < a.m ? a.n_queries : a.m;
  const int n_win = (L + a.pool_window - 1) / a.pool_window;
  const int n_sum = n_win + 1;
  unsigned short *dst = a.summaries + ((long long)b * p.n_past + np) * a.nsp * D;
  for (int item = threadIdx.x; item < a.nsp * CH; item += 256) {
    const int s = item / CH, c = item % CH;
    const int sr = s < p.g * n_sum ? s : 0;           // padding rows repeat summary 0
    const int hq = kv * p.g + sr / n_sum, w = sr % n_sum;
    int r0, r1;                                        // rows [r0, r1) of the last L rows
    if (w < n_win) {
      r0 = w * a.pool_window;
      r1 = r0 + a.pool_window < L ? r0 + a.pool_window : L;
    } else {
      r0 = L - (a.tail_avg < L ? a.tail_avg : L);
      r1 = L;
    }
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    const unsigned short *src = pv.q + ((long long)(a.m - L) * p.Hq + hq) * D + 8 * c;
    const long long stride = (long long)p.Hq * D;
#pragma unroll 4
    for (int r = r0; r < r1; ++r) {
      const uint4 x = *(const uint4 *)(src + r * stride);
      const unsigned xw[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        acc[2 * e] += __uint_as_float(xw[e] << 16);
        acc[2 * e + 1] += __uint_as_float(xw[e] & 0xffff0000u);
      }
    }
    const float inv_n = (float)(r1 - r0);
    unsigned o[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const __bf16 lo16 = (__bf16)(acc[2 * e] / inv_n), hi16 = (__bf16)(acc[2 * e + 1] / inv_n);
      o[e] = (unsigned)__builtin_bit_cast(unsigned short, lo16) | ((unsigned)__builtin_bit_cast(unsigned short, hi16) << 16);
    }
    *(uint4 *)(dst + (long long)s * D + 8 * c) = uint4{o[0], o[1], o[2], o[3]};
  }
}

// ---- scoring + per-chunk candidates.  grid (chunks, B * n_past), 4 waves; a wave scores 32 rows
//      at a time: S[summary][row] = Sigma . K^T, A = summaries (registers), B = K rows in operand
//      layout (lane = row); the lane's 16 accumulator registers are 16 summaries of its row, so
//      the maximum over summaries is local.
template <int D, int NT, int kChunkRows>  // NT = NSP / 32 summary tiles; pool rows per workgroup
__global__ __launch_bounds__(256) void retrieve_score_kernel(const Problem p, const RetrieveArgs a) {
  constexpr int NC = D / 16;
  __shared__ float sc[kChunkRows];
  __shared__ __attribute__((aligned(16))) unsigned char stage[4][32 * 2 * D];  // one K tile per wave
  const int b = blockIdx.y / p.n_past, np = blockIdx.y % p.n_past;
  const int kv = p.order[np];
  const PoolView pv = pool_view(p, a, b, kv);
  const int pool = pv.pool, lo = pv.lo;
  const int c0 = blockIdx.x * kChunkRows;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, hi = lane >> 5, col = lane & 31;
  float *cv = a.cand_val + (((long long)b * p.n_past + np) * a.n_chunks + blockIdx.x) * kMaxAnchors;
  int *ci = a.cand_idx + (((long long)b * p.n_past + np) * a.n_chunks + blockIdx.x) * kMaxAnchors;
  if (c0 >= pool || c0 + kChunkRows <= lo) {  // nothing visible in this chunk
    if (tid < kMaxAnchors) {
      cv[tid] = -INFINITY;
      ci[tid] = 0x7fffffff;
    }
    return;
  }
  const unsigned short *sg = a.summaries + ((long long)b * p.n_past + np) * a.nsp * D;
  bf16x8 A[NT][NC];  // summary (32 t + col), channels 16 kc + 8 hi .. +7
#pragma unroll
  for (int t = 0; t < NT; ++t)
#pragma unroll
    for (int kc = 0; kc < NC; ++kc) A[t][kc] = *(const bf16x8 *)(sg + (long long)(32 * t + col) * D + 16 * kc + 8 * hi);
  // K rows travel HBM -> registers with coalesced wave loads (a pool in the cache arena is
  // contiguous: 1 KB per load; rows of a token-major prompt are 2 D contiguous bytes each), are dropped into a wave-private LDS tile with the 16-byte chunks of
  // a row XOR-swizzled by the row, and come back in operand layout (lane = row).  The loads of
  // the next tile are in flight while the current one is scored.
  constexpr int RPL = 1024 / (2 * D);        // rows per 1 KB load
  constexpr int NL = 32 / RPL;               // loads per tile
  constexpr int CH = D / 8;                  // 16-byte chunks per row
  const unsigned char *kb = pv.k;
  const long long row_bytes = pv.row_bytes;
  auto swz = [](int row) { return D == 128 ? (row & 15) : ((row >> 1) & 7); };
  const long long last_byte_row = (long long)(pool - 1);
  u32x4 cur[NL], nxt[NL];
  auto fetch = [&](u32x4(&dst)[NL], int t0) {
#pragma unroll
    for (int i = 0; i < NL; ++i) {
      long long row = (long long)c0 + t0 + RPL * i + lane / CH;
      row = row < last_byte_row ? row : last_byte_row;  // clamp: stays inside the pool
      dst[i] = __builtin_nontemporal_load((const u32x4 *)(kb + row * row_bytes + (lane % CH) * 16));  // read once
    }
  };
  unsigned char *tile = stage[wave];
  fetch(cur, wave * 32);
  for (int t0 = wave * 32; t0 < kChunkRows; t0 += 128) {
    if (t0 + 128 < kChunkRows) fetch(nxt, t0 + 128);
#pragma unroll
    for (int i = 0; i < NL; ++i) {
      const int r = RPL * i + lane / CH, c = lane % CH;
      *(u32x4 *)(tile + r * (2 * D) + ((c ^ swz(r)) << 4)) = cur[i];
    }
    bf16x8 K[NC];
#pragma unroll
    for (int kc = 0; kc < NC; ++kc)
      K[kc] = *(const bf16x8 *)(tile + col * (2 * D) + (((2 * kc + hi) ^ swz(col)) << 4));
    const int row = c0 + t0 + col;
    float best = -INFINITY;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      f32x16 S = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int kc = 0; kc < NC; ++kc) S = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A[t][kc], K[kc], S, 0, 0, 0);
#pragma unroll
      for (int r = 0; r < 16; ++r) best = fmaxf(best, S[r]);
    }
    best = fmaxf(best, __shfl_xor(best, 32));  // the other 16 summaries of each tile
    if (hi == 0) sc[t0 + col] = (row >= lo && row < pool) ? best : -INFINITY;
#pragma unroll
    for (int i = 0; i < NL; ++i) cur[i] = nxt[i];
  }
  __syncthreads();
  // The chunk's best n_anchors rows, in order.  Every thread owns kChunkRows/256 scores.  Each wave
  // first finds the best n_anchors of its own quarter (rounds of a wave-wide arg-max by shuffles,
  // the winner's owner retires it: no workgroup barrier), then the first wave merges the four
  // sorted lists (lane w < 4 holds the head of list w).
  float mine[kChunkRows / 256];
#pragma unroll
  for (int e = 0; e < kChunkRows / 256; ++e) mine[e] = sc[tid + 256 * e];
  __shared__ float wl_v[4][kMaxAnchors];
  __shared__ int wl_i[4][kMaxAnchors];
  for (int r = 0; r < a.n_anchors; ++r) {
    float bv = -INFINITY;
    int bi = 0x7fffffff;
#pragma unroll
    for (int e = 0; e < kChunkRows / 256; ++e)
      if (better(mine[e], c0 + tid + 256 * e, bv, bi)) {
        bv = mine[e];
        bi = c0 + tid + 256 * e;
      }
    float v = bv;
    int i = bi;
    wave_best(v, i);
    if (lane == 0) {
      wl_v[wave][r] = v;
      wl_i[wave][r] = v == -INFINITY ? 0x7fffffff : i;
    }
    if (v != -INFINITY && bi == i) {  // this lane owns the winner
      const int off = i - c0;
#pragma unroll
      for (int e = 0; e < kChunkRows / 256; ++e)
        if (e == off / 256) mine[e] = -INFINITY;
    }
  }
  __syncthreads();
  if (tid < 64) {
    int hp = 0;
    const bool list = tid < 4 && a.n_anchors > 0;
    float hv = list ? wl_v[tid][0] : -INFINITY;
    int hr = list ? wl_i[tid][0] : 0x7fffffff;
    for (int r = 0; r < a.n_anchors; ++r) {
      float v = hv;
      int i = hr;
#pragma unroll
      for (int sh = 2; sh >= 1; sh >>= 1) {  // the four heads sit in lanes 0..3
        const float w = __shfl_xor(v, sh);
        const int j = __shfl_xor(i, sh);
        if (better(w, j, v, i)) {
          v = w;
          i = j;
        }
      }
      v = __shfl(v, 0);
      i = __shfl(i, 0);
      if (tid == 0) {
        cv[r] = v;
        ci[r] = v == -INFINITY ? 0x7fffffff : i;
      }
      if (list && v != -INFINITY && hr == i) {
        hp += 1;
        const bool more = hp < a.n_anchors;
        hv = more ? wl_v[tid][more ? hp : 0] : -INFINITY;
        hr = more ? wl_i[tid][more ? hp : 0] : 0x7fffffff;
      }
    }
  }
}

// ---- merge the candidates of all chunks, expand, pad, emit.  One workgroup per (b, PAST head).
// The chosen rows are kept as sorted, disjoint, merged row ranges, one per lane of wave 0 (at
// most one range per anchor window plus the padding prefix); the expansion itself is sequential
// in the anchors' score order, but every step on the range list is a constant number of
// wave-wide operations (ballot to locate, shuffle to insert or delete).
constexpr int kCandLds = 4096;  // candidates held in LDS; beyond that they are re-read from memory

__global__ __launch_bounds__(256) void retrieve_select_kernel(const Problem p, const RetrieveArgs a) {
  __shared__ float sm_v[4];
  __shared__ int sm_i[4];
  __shared__ int anchors[kMaxAnchors];
  __shared__ float lc_v[kCandLds];
  __shared__ int lc_i[kCandLds];
  __shared__ int p_lo[64], p_before[65];
  __shared__ int n_pieces;
  const int b = blockIdx.x / p.n_past, np = blockIdx.x % p.n_past;
  const int kv = p.order[np];
  const PoolView pv = pool_view(p, a, b, kv);
  const int pool = pv.pool, lo = pv.lo;
  const int tid = threadIdx.x;
  const long long base = ((long long)b * p.n_past + np) * a.n_chunks * kMaxAnchors;
  // live candidates: n_anchors per chunk
  const int n_cand = a.n_chunks * a.n_anchors;
  const bool in_lds = n_cand <= kCandLds;
  if (in_lds)
    for (int c = tid; c < n_cand; c += 256) {
      const long long src = base + (long long)(c / a.n_anchors) * kMaxAnchors + c % a.n_anchors;
      lc_v[c] = a.cand_val[src];
      lc_i[c] = a.cand_idx[src];
    }
  __syncthreads();
  // anchors: the n_anchors best candidates (value desc, row asc)
  int n_anch = 0;
  constexpr int kHeads = 4;  // chunk lists per lane in the single-wave merge
  if (in_lds && a.n_chunks <= 64 * kHeads) {
    // Every chunk's list is already sorted (the score kernel emits its winners in order), so the
    // global order is a merge of sorted lists: one wave, lane l owns the lists of chunks
    // l, l+64, ... and keeps their heads in registers; a round takes the best head over the wave
    // and only the owning lane moves that list on.  No workgroup barrier in the loop.
    if (tid < 64) {
      float hv[kHeads];
      int hr[kHeads], hp[kHeads];
#pragma unroll
      for (int k = 0; k < kHeads; ++k) {
        const int ch = tid + 64 * k;
        const bool ok = ch < a.n_chunks && a.n_anchors > 0;
        hp[k] = 0;
        hv[k] = ok ? lc_v[ch * a.n_anchors] : -INFINITY;
        hr[k] = ok ? lc_i[ch * a.n_anchors] : 0x7fffffff;
      }
      for (int r = 0; r < a.n_anchors; ++r) {
        float bv = hv[0];
        int bi = hr[0], bk = 0;
#pragma unroll
        for (int k = 1; k < kHeads; ++k)
          if (better(hv[k], hr[k], bv, bi)) {
            bv = hv[k];
            bi = hr[k];
            bk = k;
          }
        float v = bv;
        int i = bi;
        wave_best(v, i);
        if (v == -INFINITY) break;
        if (tid == 0) anchors[r] = i;
        n_anch = r + 1;
        if (bv == v && bi == i) {  // rows are unique over the chunks: exactly one lane owns the winner
#pragma unroll
          for (int k = 0; k < kHeads; ++k)
            if (k == bk) {
              hp[k] += 1;
              const int src = (tid + 64 * k) * a.n_anchors + hp[k];
              const bool more = hp[k] < a.n_anchors;
              hv[k] = more ? lc_v[more ? src : 0] : -INFINITY;
              hr[k] = more ? lc_i[more ? src : 0] : 0x7fffffff;
            }
        }
      }
    }
  } else {
    // many chunks: n_anchors rounds of a workgroup-wide arg-max over all candidates; a candidate
    // is retired by remembering the last winner: the order is total, so "strictly after the last
    // winner" selects the next one without writing anything
    float last_v = INFINITY;
    int last_i = -1;
    for (int r = 0; r < a.n_anchors; ++r) {
      float v = -INFINITY;
      int i = 0x7fffffff;
      for (int c = tid; c < n_cand; c += 256) {
        float w;
        int j;
        if (in_lds) {
          w = lc_v[c];
          j = lc_i[c];
        } else {
          const long long src = base + (long long)(c / a.n_anchors) * kMaxAnchors + c % a.n_anchors;
          w = a.cand_val[src];
          j = a.cand_idx[src];
        }
        if (w == -INFINITY) continue;
        if (better(w, j, last_v, last_i) || (w == last_v && j == last_i)) continue;  // taken already
        if (better(w, j, v, i)) {
          v = w;
          i = j;
        }
      }
      block_best(v, i, sm_v, sm_i);
      if (v == -INFINITY) break;
      if (tid == 0) anchors[r] = i;
      last_v = v;
      last_i = i;
      n_anch = r + 1;
    }
  }
  __syncthreads();  // anchors[] is complete (the first wave uses it below)
  const int visible = pool - lo;
  const int want = a.R < visible ? a.R : visible;
  if (tid < 64) {
    const int lane = tid;
    int plo = 0x7fffffff, phi = 0x7fffffff;  // range `lane` of the sorted list (unused lanes: +inf)
    int n = 0, count = 0;
    auto add_range = [&](int s, int e) {  // rows of [s, e) not yet in, ascending, until `want`
      int cur = s;
      while (cur < e && count < want) {
        const unsigned long long inside = __builtin_amdgcn_ballot_w64(plo <= cur && cur < phi);
        if (inside) {  // cur lies in a range: continue behind it
          cur = __builtin_amdgcn_readlane(phi, (int)__builtin_ctzll(inside));
          continue;
        }
        const unsigned long long later = __builtin_amdgcn_ballot_w64(lane < n && plo > cur);
        const int kn = later ? (int)__builtin_ctzll(later) : n;  // first range behind cur
        int next_start = e;
        if (later) {
          const int ns = __builtin_amdgcn_readlane(plo, kn);
          next_start = ns < e ? ns : e;
        }
        int take = next_start - cur;
        if (take > want - count) take = want - count;
        int j;  // the range that now ends at cur + take
        if (kn > 0 && __builtin_amdgcn_readlane(phi, kn - 1) == cur) {  // grows the range before it
          j = kn - 1;
          if (lane == j) phi = cur + take;
        } else {  // new range at position kn: ranges kn.. move up one lane
          const int ulo = __shfl_up(plo, 1), uhi = __shfl_up(phi, 1);
          if (lane > kn) {
            plo = ulo;
            phi = uhi;
          } else if (lane == kn) {
            plo = cur;
            phi = cur + take;
          }
          j = kn;
          n += 1;
        }
        if (j + 1 < n && __builtin_amdgcn_readlane(plo, j + 1) == cur + take) {  // touches the next: merge
          const int nhi = __builtin_amdgcn_readlane(phi, j + 1);
          const int dlo = __shfl_down(plo, 1), dhi = __shfl_down(phi, 1);
          if (lane == j) phi = nhi;
          else if (lane > j) {
            plo = lane + 1 < 64 ? dlo : 0x7fffffff;
            phi = lane + 1 < 64 ? dhi : 0x7fffffff;
          }
          n -= 1;
        }
        count += take;
        cur += take;
      }
    };
    for (int r = 0; r < n_anch; ++r) {
      const int an = anchors[r];
      const int s = an - a.win_before > lo ? an - a.win_before : lo;
      const int e = an + a.win_after + 1 < pool ? an + a.win_after + 1 : pool;
      add_range(s, e);
    }
    add_range(lo, pool);  // padding: the earliest visible rows not yet in
    // rows before each range (exclusive prefix sum of the lengths)
    int len = lane < n ? phi - plo : 0, incl = len;
#pragma unroll
    for (int sh = 1; sh < 64; sh <<= 1) {
      const int up = __shfl_up(incl, sh);
      if (lane >= sh) incl += up;
    }
    p_lo[lane] = plo;
    p_before[lane] = incl - len;
    if (lane == 63) p_before[64] = incl;
    if (lane == 0) n_pieces = n;
  }
  __syncthreads();
  int *out = a.idx_out + ((long long)b * p.n_past + np) * a.R;
  const int total = p_before[64];
  for (int o = tid; o < a.R; o += 256) {
    int val = 0;
    if (o < total) {
      int k = 0;
      while (k + 1 < n_pieces && p_before[k + 1] <= o) ++k;
      val = p_lo[k] + (o - p_before[k]);
    } else if (total > 0) {
      val = pool - 1;  // unreachable when R <= visible rows (checked on the host)
    }
    out[o] = val;
  }
}

hipError_t launch_retrieve(const Problem &p, const RetrieveArgs &a, hipStream_t st) {
  const int seqs = a.k_seq ? p.B * a.n_seg : p.B;  // whole-prompt form: one "sequence" per (b, segment)
  const dim3 heads(seqs * p.n_past);
  if (p.D == 128) hipLaunchKernelGGL(retrieve_summaries_kernel<128>, heads, dim3(256), 0, st, p, a);
  else hipLaunchKernelGGL(retrieve_summaries_kernel<64>, heads, dim3(256), 0, st, p, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const dim3 grid(a.n_chunks, seqs * p.n_past);
  const int nt = a.nsp / 32;
#define SEGATTN_SCORE(DD, NTT)                                                                            \
  do {                                                                                                    \
    if (a.chunk_rows == 512) hipLaunchKernelGGL((retrieve_score_kernel<DD, NTT, 512>), grid, dim3(256), 0, st, p, a); \
    else if (a.chunk_rows == 1024) hipLaunchKernelGGL((retrieve_score_kernel<DD, NTT, 1024>), grid, dim3(256), 0, st, p, a); \
    else hipLaunchKernelGGL((retrieve_score_kernel<DD, NTT, 4096>), grid, dim3(256), 0, st, p, a);         \
  } while (0)
  if (p.D == 128) {
    if (nt == 1) SEGATTN_SCORE(128, 1);
    else SEGATTN_SCORE(128, 2);
  } else {
    if (nt == 1) SEGATTN_SCORE(64, 1);
    else SEGATTN_SCORE(64, 2);
  }
#undef SEGATTN_SCORE
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(retrieve_select_kernel, heads, dim3(256), 0, st, p, a);
  return hipGetLastError();
}

}  // namespace segattn
