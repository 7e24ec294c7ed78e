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
//                        de-duplicate, keep the best" yields.)  Two levels: every 4096-row chunk
//                        keeps its own best n_anchors next to the scores in LDS -- scores never
//                        go to HBM -- and one workgroup per head merges the candidates
//   window expansion     anchors in descending score order add rows a - win_before .. a + win_after
//                        (clipped to the visible pool, ascending, rows already in skipped) until
//                        R rows are in; then the earliest visible rows pad to R; sorted output
#include "segattn_internal.h"

namespace segattn {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kChunkRows = 4096;   // pool rows per scoring workgroup
constexpr int kMaxAnchors = 32;
constexpr int kMaxPieces = 160;    // disjoint row ranges of one result

__device__ inline const int *rmeta(const unsigned char *cache, const CacheGeom &g, const Problem &p, int b, int h) {
  return (const int *)(cache + g.meta_off) + ((long long)b * p.Hkv + h) * kMetaInts;
}

// (value, row) pairs ordered by value descending, then row ascending
__device__ inline bool better(float v, int i, float w, int j) { return v > w || (v == w && i < j); }

// Workgroup-wide best (value, row); every thread gets the result.  sm: 2 * 4 words of LDS.
__device__ inline void block_best(float &v, int &i, float *sm_v, int *sm_i) {
#pragma unroll
  for (int sh = 32; sh >= 1; sh >>= 1) {
    const float w = __shfl_xor(v, sh);
    const int j = __shfl_xor(i, sh);
    if (better(w, j, v, i)) {
      v = w;
      i = j;
    }
  }
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
  const int b = blockIdx.x / p.n_past, np = blockIdx.x % p.n_past;
  const int kv = p.order[np];
  const int L = a.n_queries < a.m ? a.n_queries : a.m;
  const int n_win = (L + a.pool_window - 1) / a.pool_window;
  const int n_sum = n_win + 1;
  unsigned short *dst = a.summaries + ((long long)b * p.n_past + np) * a.nsp * D;
  for (int item = threadIdx.x; item < a.nsp * D; item += 256) {
    const int s = item / D, d = item % D;
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
    float acc = 0.f;
    for (int r = r0; r < r1; ++r)
      acc += __uint_as_float((unsigned)a.q_prev[(((long long)b * a.m + (a.m - L + r)) * p.Hq + hq) * D + d] << 16);
    dst[item] = __builtin_bit_cast(unsigned short, (__bf16)(acc / (float)(r1 - r0)));
  }
}

// ---- scoring + per-chunk candidates.  grid (chunks, B * n_past), 4 waves; a wave scores 32 rows
//      at a time: S[summary][row] = Sigma . K^T, A = summaries (registers), B = K rows straight
//      from HBM in operand layout (lane = row, 16-byte pieces); the lane's 16 accumulator
//      registers are 16 summaries of its row, so the maximum over summaries is local.
template <int D, int NT>  // NT = NSP / 32 summary tiles
__global__ __launch_bounds__(256) void retrieve_score_kernel(const Problem p, const RetrieveArgs a) {
  constexpr int NC = D / 16;
  __shared__ float sc[kChunkRows];
  __shared__ float sm_v[4];
  __shared__ int sm_i[4];
  const int b = blockIdx.y / p.n_past, np = blockIdx.y % p.n_past;
  const int kv = p.order[np];
  const int *meta = rmeta(a.cache, a.geom, p, b, kv);
  const int pool = meta[META_POOL], lo = meta[META_LO];
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
  const unsigned short *kb = (const unsigned short *)(a.cache + k_block_off(p, a.geom, b, kv));
  for (int t0 = wave * 32; t0 < kChunkRows; t0 += 128) {
    const int row = c0 + t0 + col;
    const int rc = row < pool ? row : pool - 1;  // clamp: stays inside the pool
    bf16x8 K[NC];
#pragma unroll
    for (int kc = 0; kc < NC; ++kc) K[kc] = *(const bf16x8 *)(kb + (long long)rc * D + 16 * kc + 8 * hi);
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
  }
  __syncthreads();
  // the chunk's best n_anchors rows: every thread owns 16 scores; n_anchors rounds of a
  // workgroup-wide arg-max, the winner's owner retires it
  float mine[kChunkRows / 256];
#pragma unroll
  for (int e = 0; e < kChunkRows / 256; ++e) mine[e] = sc[tid + 256 * e];
  for (int r = 0; r < a.n_anchors; ++r) {
    float v = -INFINITY;
    int i = 0x7fffffff;
#pragma unroll
    for (int e = 0; e < kChunkRows / 256; ++e)
      if (better(mine[e], c0 + tid + 256 * e, v, i)) {
        v = mine[e];
        i = c0 + tid + 256 * e;
      }
    block_best(v, i, sm_v, sm_i);
    if (tid == 0) {
      cv[r] = v;
      ci[r] = v == -INFINITY ? 0x7fffffff : i;
    }
    const int off = i - c0;
    if (v != -INFINITY && (off & 255) == tid) {
#pragma unroll
      for (int e = 0; e < kChunkRows / 256; ++e)
        if (e == off / 256) mine[e] = -INFINITY;
    }
  }
}

// ---- merge the candidates of all chunks, expand, pad, emit.  One workgroup per (b, PAST head).
__global__ __launch_bounds__(256) void retrieve_select_kernel(const Problem p, const RetrieveArgs a) {
  __shared__ float sm_v[4];
  __shared__ int sm_i[4];
  __shared__ int anchors[kMaxAnchors];
  __shared__ int p_lo[kMaxPieces], p_hi[kMaxPieces], p_before[kMaxPieces + 1];
  __shared__ int n_pieces;
  const int b = blockIdx.x / p.n_past, np = blockIdx.x % p.n_past;
  const int kv = p.order[np];
  const int *meta = rmeta(a.cache, a.geom, p, b, kv);
  const int pool = meta[META_POOL], lo = meta[META_LO];
  const int tid = threadIdx.x;
  const long long base = ((long long)b * p.n_past + np) * a.n_chunks * kMaxAnchors;
  const int n_cand = a.n_chunks * kMaxAnchors;
  // anchors: n_anchors rounds of arg-max over the candidates (value desc, row asc); a candidate
  // is retired by remembering the last winner: the order is total, so "strictly after the last
  // winner" selects the next one without writing anything
  float last_v = INFINITY;
  int last_i = -1;
  int n_anch = 0;
  for (int r = 0; r < a.n_anchors; ++r) {
    float v = -INFINITY;
    int i = 0x7fffffff;
    for (int c = tid; c < n_cand; c += 256) {
      if ((c % kMaxAnchors) >= a.n_anchors) continue;
      const float w = a.cand_val[base + c];
      const int j = a.cand_idx[base + c];
      if (w == -INFINITY) continue;
      if (better(w, j, last_v, last_i)) continue;  // already taken (or is the last winner's better)
      if (w == last_v && j == last_i) continue;
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
  __syncthreads();
  const int visible = pool - lo;
  const int want = a.R < visible ? a.R : visible;
  if (tid == 0) {
    // pieces: disjoint row ranges kept sorted by start
    int np_ = 0, count = 0;
    auto insert = [&](int s, int e) {  // insert [s, e) keeping the list sorted
      int k = np_;
      while (k > 0 && p_lo[k - 1] > s) {
        p_lo[k] = p_lo[k - 1];
        p_hi[k] = p_hi[k - 1];
        --k;
      }
      p_lo[k] = s;
      p_hi[k] = e;
      ++np_;
    };
    auto add_range = [&](int s, int e) {  // rows of [s, e) not yet in, ascending, until `want`
      int cur = s;
      while (cur < e && count < want && np_ < kMaxPieces) {
        // skip over a piece that contains cur
        int k = 0;
        bool inside = false;
        int next_start = e;
        for (k = 0; k < np_; ++k) {
          if (p_lo[k] <= cur && cur < p_hi[k]) {
            inside = true;
            break;
          }
          if (p_lo[k] > cur) {
            next_start = p_lo[k] < e ? p_lo[k] : e;
            break;
          }
        }
        if (inside) {
          cur = p_hi[k];
          continue;
        }
        int take = next_start - cur;
        if (take > want - count) take = want - count;
        insert(cur, cur + take);
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
    int before = 0;
    for (int k = 0; k < np_; ++k) {
      p_before[k] = before;
      before += p_hi[k] - p_lo[k];
    }
    p_before[np_] = before;
    n_pieces = np_;
  }
  __syncthreads();
  int *out = a.idx_out + ((long long)b * p.n_past + np) * a.R;
  const int total = p_before[n_pieces];
  for (int o = tid; o < a.R; o += 256) {
    int val = 0;
    if (o < total) {
      int k = 0;
      while (k + 1 < n_pieces && p_before[k + 1] <= o) ++k;
      val = p_lo[k] + (o - p_before[k]);
    } else if (total > 0) {
      val = p_hi[n_pieces - 1] - 1;  // unreachable when R <= visible rows (checked on the host)
    }
    out[o] = val;
  }
}

hipError_t launch_retrieve(const Problem &p, const RetrieveArgs &a, hipStream_t st) {
  const dim3 heads(p.B * p.n_past);
  if (p.D == 128) hipLaunchKernelGGL(retrieve_summaries_kernel<128>, heads, dim3(256), 0, st, p, a);
  else hipLaunchKernelGGL(retrieve_summaries_kernel<64>, heads, dim3(256), 0, st, p, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const dim3 grid(a.n_chunks, p.B * p.n_past);
  const int nt = a.nsp / 32;
  if (p.D == 128) {
    if (nt == 1) hipLaunchKernelGGL((retrieve_score_kernel<128, 1>), grid, dim3(256), 0, st, p, a);
    else hipLaunchKernelGGL((retrieve_score_kernel<128, 2>), grid, dim3(256), 0, st, p, a);
  } else {
    if (nt == 1) hipLaunchKernelGGL((retrieve_score_kernel<64, 1>), grid, dim3(256), 0, st, p, a);
    else hipLaunchKernelGGL((retrieve_score_kernel<64, 2>), grid, dim3(256), 0, st, p, a);
  }
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(retrieve_select_kernel, heads, dim3(256), 0, st, p, a);
  return hipGetLastError();
}

}  // namespace segattn
