// bf16 MFMA backward of segment-level attention for gfx950 (training with truncated
// backpropagation over segments, Sec. 3.2).  Two kernels, no atomics, deterministic:
//
//   bwd_dq_kernel    a wave owns 32 query rows of one head and walks the keys it sees in steps of
//                    32 (prefix span, then its own segment up to the diagonal):
//                      S^T  = K . Q^T          P^T = exp2(S^T c - LSE)
//                      dP^T = V . dO^T         dS^T = P^T (dP^T - delta)
//                      dQ^T += K^T . dS^T      (every visible key contributes, past rows too)
//   bwd_dkv_kernel   a wave owns 32 key rows of one KV head and walks the queries whose pair with
//                    them is differentiable (same segment from the diagonal on; the next segment
//                    if the keys are in its carried tail), for each query head of the group:
//                      S  = Q . K^T            P  = exp2(S c - LSE)
//                      dP = dO . V^T           dS = P (dP - delta)
//                      dV^T += dO^T . P        dK^T += Q^T . dS
//                    Rows a query reaches only through the PAST bit are forward-only (no-gradient
//                    lemma, Appendix B): they never show up here.
//
// As in the forward kernel the products are arranged so that the accumulator layout of the
// score tile (lane = its column, the lane's 16 registers = rows) is the B-operand layout of
// the products that consume P and dS; the transposed A operands (K^T, dO^T, Q^T) come from
// row-major LDS tiles with ds_read_b64_tr_b16.  Tiles are staged HBM -> registers -> LDS,
// double-buffered, one barrier per step; the 16-byte chunks of a row are XOR-swizzled against
// bank conflicts.
// This file is compiled with the compiler's default MFMA register form (accumulators in
// accumulation registers, placed by the register allocator); all products are builtins, so the
// compiler tracks every MFMA hazard itself.
#include <string.h>

#include "segattn_work.h"

namespace segattn {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
#define LDS_AS __attribute__((address_space(3)))

constexpr int kBwdStep = 32;
constexpr float kLog2e = 1.4426950408889634f;

// A [32 x D] bf16 tile in LDS: dense rows, the 16-byte chunks of a row XOR-swizzled with a
// function of the row chosen so that both access patterns are free of bank conflicts: the row
// reads (16 lanes = 16 consecutive rows at one logical chunk) and the transposing reads (16
// lanes = 4 consecutive rows x 32 contiguous bytes).
template <int D>
struct BwdTile {
  static constexpr int kRowBytes = 2 * D;
  static constexpr int kBytes = kBwdStep * kRowBytes;
  static constexpr int kChunks = D / 8;                 // 16-byte chunks per row
  static constexpr int kLoads = kBwdStep * kChunks / 256;  // chunks per thread per tile
  __device__ static constexpr int swz(int row) {
    if (D == 128) return ((row & 3) << 2) | ((row >> 2) & 3);
    const int a = row >> 1;  // 128-byte rows: two rows share a 64-bank line
    return ((a & 1) << 2) | (((a >> 2) & 1) << 1) | ((a >> 1) & 1);
  }
  // byte offset of logical chunk `chunk` of row `row`
  __device__ static constexpr int at(int row, int chunk) { return row * kRowBytes + ((chunk ^ swz(row)) << 4); }
};

// acc += A . B
__device__ inline void mma_acc(f32x16 &acc, const bf16x8 a, const bf16x8 b) {
  acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc, 0, 0, 0);
}

// Move four dwords into accumulation registers; the result is used as an MFMA operand only.
__device__ inline bf16x8 park(const uint4 v) {
  int a0, a1, a2, a3;
  asm volatile("v_accvgpr_write_b32 %0, %1" : "=a"(a0) : "v"(v.x));
  asm volatile("v_accvgpr_write_b32 %0, %1" : "=a"(a1) : "v"(v.y));
  asm volatile("v_accvgpr_write_b32 %0, %1" : "=a"(a2) : "v"(v.z));
  asm volatile("v_accvgpr_write_b32 %0, %1" : "=a"(a3) : "v"(v.w));
  typedef int i32x4 __attribute__((ext_vector_type(4)));
  const i32x4 q4 = {a0, a1, a2, a3};
  return __builtin_bit_cast(bf16x8, q4);
}

// A operand of a transposed product from a row-major [32 x D] tile: for the 32-column block nb
// and the 16-row half h2, k-slot e of half-wave hi is tile row 16 h2 + 8 (e/4) + 4 hi + e%4 (the
// accumulator layout of the score tile) and the lane's operand row is tile column 32 nb + lane%32.
template <int D>
__device__ inline bf16x8 read_transposed(const unsigned char *tile, int lane, int nb, int h2) {
  using T = BwdTile<D>;
  const int hi = lane >> 5, i16 = lane & 15, g16 = (lane >> 4) & 1;
  const int row = 4 * hi + (i16 >> 2) + 16 * h2;
  const int chunk = 4 * nb + 2 * g16 + ((i16 & 3) >> 1), half = 8 * (i16 & 1);
  const LDS_AS s16x4 *p0 = (const LDS_AS s16x4 *)(tile + T::at(row, chunk) + half);
  const LDS_AS s16x4 *p1 = (const LDS_AS s16x4 *)(tile + T::at(row + 8, chunk) + half);
  const s16x4 a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4 *)p0);
  const s16x4 b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4 *)p1);
  return __builtin_bit_cast(bf16x8, __builtin_shufflevector(a, b, 0, 1, 2, 3, 4, 5, 6, 7));
}

// A operand of a row product: tile row lane%32, elements 16 kc + 8 (lane/32) .. +7
template <int D>
__device__ inline bf16x8 read_row(const unsigned char *tile, int lane, int kc) {
  using T = BwdTile<D>;
  return *(const bf16x8 *)(tile + T::at(lane & 31, 2 * kc + (lane >> 5)));
}

// Cooperative copy of rows [r0, r0+32) (clamped to r_last) of a row-major bf16 matrix with
// `stride` elements between rows: global -> registers, registers -> LDS tile.
template <int D>
struct TileRegs {
  uint4 x[BwdTile<D>::kLoads];
};
template <int D>
__device__ inline TileRegs<D> tile_fetch(const unsigned short *base, long long stride, long long r0,
                                         long long r_last, int tid) {
  using T = BwdTile<D>;
  TileRegs<D> t;
#pragma unroll
  for (int i = 0; i < T::kLoads; ++i) {
    const int c = tid + 256 * i;
    long long r = r0 + c / T::kChunks;
    r = r < r_last ? r : r_last;
    t.x[i] = *(const uint4 *)(base + r * stride + (c % T::kChunks) * 8);
  }
  return t;
}
template <int D>
__device__ inline void tile_store(const TileRegs<D> &t, unsigned char *tile, int tid) {
  using T = BwdTile<D>;
#pragma unroll
  for (int i = 0; i < T::kLoads; ++i) {
    const int c = tid + 256 * i;
    *(uint4 *)(tile + T::at(c / T::kChunks, c % T::kChunks)) = t.x[i];
  }
}

// ---------------------------------------------------------------------------------------------
// dQ
// ---------------------------------------------------------------------------------------------
template <int D, int HS>
__global__ __launch_bounds__(256, 1) void bwd_dq_kernel(const Problem p, const PrefillArgs pa, const BwdArgs a) {
  using T = BwdTile<D>;
  constexpr int NC = D / 16, NB = D / 32;
  constexpr int RW = 32;             // query rows per wave
  constexpr int BQ = (4 / HS) * RW;  // query rows per workgroup
  __shared__ __attribute__((aligned(16))) unsigned char smem[2][2][T::kBytes];  // [buffer][K,V]

  const WorkItem w = resolve(p, pa, blockIdx.x, BQ, HS);
  if (!w.valid) return;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int hi = lane >> 5, col = lane & 31;
  const int head = w.kv * p.g + w.hsub * HS + (wave % HS);
  const int tw0 = w.t0 + (wave / HS) * RW;
  const int last_row = w.n1 - 1;
  const float c = p.scale_log2e;
  // global row of the segment's first token (b*N + s) and this lane's query row
  const long long seg_row = (w.q - a.q) / ((long long)p.Hq * D);
  int t = tw0 + col;
  const bool row_ok = t <= last_row;
  t = row_ok ? t : last_row;
  const long long qoff = ((seg_row + t) * p.Hq + head) * D;
  const long long stat = (w.lse - a.lse) + (long long)head * a.n + t;  // index into lse / delta
  const float lse2 = a.lse[stat] * kLog2e, delta = a.delta[stat];

  bf16x8 Qr[NC], Gr[NC];  // Q^T and dO^T operands: row `col`, elements 16 kc + 8 hi .. +7
#pragma unroll
  for (int kc = 0; kc < NC; ++kc) {
    Qr[kc] = *(const bf16x8 *)(a.q + qoff + 16 * kc + 8 * hi);
    Gr[kc] = *(const bf16x8 *)(a.dout + qoff + 16 * kc + 8 * hi);
  }
  f32x16 acc[NB];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[nb][r] = 0.f;

  const int n1_needed = (w.t0 + BQ < w.n1) ? (w.t0 + BQ) : w.n1;
  const int nst0 = (w.n0 + kBwdStep - 1) / kBwdStep;
  const int nst1 = (n1_needed + kBwdStep - 1) / kBwdStep;
  const int nsteps = nst0 + nst1;
  const int my_last = tw0 + RW - 1;  // keys of the own segment beyond this row are invisible to the wave

  // tiles of step j (clamped to the last step, whose re-fetch is not used)
  auto fetch_k = [&](int j) {
    j = j < nsteps ? j : nsteps - 1;
    const bool s1 = j >= nst0;
    return tile_fetch<D>(s1 ? w.k1 : w.k0, s1 ? w.stride1 : w.stride0, (long long)(s1 ? j - nst0 : j) * kBwdStep,
                         (s1 ? w.n1 : w.n0) - 1, tid);
  };
  auto fetch_v = [&](int j) {
    j = j < nsteps ? j : nsteps - 1;
    const bool s1 = j >= nst0;
    return tile_fetch<D>(s1 ? w.v1 : w.v0, s1 ? w.stride1 : w.stride0, (long long)(s1 ? j - nst0 : j) * kBwdStep,
                         (s1 ? w.n1 : w.n0) - 1, tid);
  };
  {
    const TileRegs<D> kr = fetch_k(0), vr = fetch_v(0);
    tile_store<D>(kr, smem[0][0], tid);
    tile_store<D>(vr, smem[0][1], tid);
  }
  __syncthreads();
  (void)my_last;
  for (int j = 0; j < nsteps; ++j) {
    const int cur = j & 1;
    const TileRegs<D> kr = fetch_k(j + 1), vr = fetch_v(j + 1);
    const bool own = j >= nst0;
    const int k0 = (own ? j - nst0 : j) * kBwdStep;           // first key of the step inside its span
    const int span_len = own ? w.n1 : w.n0;
    {
      const unsigned char *kt = smem[cur][0], *vt = smem[cur][1];
      f32x16 S = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
      f32x16 dP = S;
#pragma unroll
      for (int kc = 0; kc < NC; ++kc) {
        S = __builtin_amdgcn_mfma_f32_32x32x16_bf16(read_row<D>(kt, lane, kc), Qr[kc], S, 0, 0, 0);
        dP = __builtin_amdgcn_mfma_f32_32x32x16_bf16(read_row<D>(vt, lane, kc), Gr[kc], dP, 0, 0, 0);
      }
      bf16x8 dS[2];
      const int kmax = own ? (t < span_len - 1 ? t : span_len - 1) : span_len - 1;  // last visible key of the span
#pragma unroll
      for (int h2 = 0; h2 < 2; ++h2) {
        f32x8 e;
#pragma unroll
        for (int x = 0; x < 8; ++x) {
          const int r = 8 * h2 + x;
          const int key = k0 + 8 * (r / 4) + 4 * hi + r % 4;
          // a masked pair gets exponent -inf: its weight is exactly 0, without a branch
          const float pr = __builtin_amdgcn_exp2f(key <= kmax ? fmaf(S[r], c, -lse2) : -INFINITY);
          e[x] = pr * (dP[r] - delta);
        }
        dS[h2] = __builtin_convertvector(e, bf16x8);
      }
#pragma unroll
      for (int h2 = 0; h2 < 2; ++h2)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) mma_acc(acc[nb], read_transposed<D>(kt, lane, nb, h2), dS[h2]);
    }
    tile_store<D>(kr, smem[cur ^ 1][0], tid);
    tile_store<D>(vr, smem[cur ^ 1][1], tid);
    __syncthreads();
  }
  if (!row_ok) return;
  // dQ^T[d][q]: this lane holds, for its query row, d = 32 nb + 8 rg + 4 hi .. +3
#pragma unroll
  for (int nb = 0; nb < NB; ++nb)
#pragma unroll
    for (int rg = 0; rg < 4; ++rg) {
      const int d = 32 * nb + 8 * rg + 4 * hi;
      const f32x4 o = {acc[nb][4 * rg + 0] * p.scale, acc[nb][4 * rg + 1] * p.scale,
                       acc[nb][4 * rg + 2] * p.scale, acc[nb][4 * rg + 3] * p.scale};
      if (p.out_fp32) *(f32x4 *)((float *)a.dq + qoff + d) = o;
      else *(uint2 *)((unsigned short *)a.dq + qoff + d) = __builtin_bit_cast(uint2, __builtin_convertvector(o, bf16x4));
    }
}

// ---------------------------------------------------------------------------------------------
// dK, dV
// ---------------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(256, 1) void bwd_dkv_kernel(const Problem p, const BwdArgs a, const int blocks_per_seg,
                                                         const int n_seg) {
  using T = BwdTile<D>;
  constexpr int NC = D / 16, NB = D / 32;
  constexpr int BK = 128;  // key rows per workgroup
  __shared__ __attribute__((aligned(16))) unsigned char smem[2][2][T::kBytes];  // [buffer][Q,dO]
  __shared__ __attribute__((aligned(16))) float stats[2][2][kBwdStep];                                       // [buffer][lse*log2e, delta]

  // blockIdx -> (key block inside its segment, segment, kv head, b); blocks near the start of a
  // segment have the most queries after them and come first
  const int per = n_seg * p.Hkv * p.B;
  const int kb = blockIdx.x / per;
  int rest = blockIdx.x % per;
  const int seg = rest % n_seg;
  rest /= n_seg;
  const int kv = rest % p.Hkv;
  const int b = rest / p.Hkv;
  const int pol = p.policy[kv];
  const long long N = a.n;
  const long long s0 = (long long)seg * p.S;
  const long long seg_end = s0 + p.S < N ? s0 + p.S : N;
  const long long j0 = s0 + (long long)kb * BK;
  if (j0 >= seg_end) return;
  const long long j_end = j0 + BK < seg_end ? j0 + BK : seg_end;  // keys of the workgroup: [j0, j_end)

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int hi = lane >> 5, col = lane & 31;
  const float c = p.scale_log2e;
  // this lane's key row (clamped for loads; stores are guarded)
  const long long jw0 = j0 + 32 * wave;
  long long jk = jw0 + col;
  const bool key_ok = jk < j_end;
  jk = key_ok ? jk : j_end - 1;
  const long long koff = ((b * N + jk) * p.Hkv + kv) * D;
  // K^T and V^T operands of this lane's key: only ever MFMA operands, so they are parked in
  // accumulation registers and the vector registers stay free for operand prefetch
  bf16x8 Kr[NC], Vr[NC];
#pragma unroll
  for (int kc = 0; kc < NC; ++kc) {
    Kr[kc] = park(*(const uint4 *)(a.k + koff + 16 * kc + 8 * hi));
    Vr[kc] = park(*(const uint4 *)(a.v + koff + 16 * kc + 8 * hi));
  }
  f32x16 dKa[NB], dVa[NB];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      dKa[nb][r] = 0.f;
      dVa[nb][r] = 0.f;
    }

  // queries: own segment from row j0 on; then, for keys in the carried tail of the next segment,
  // all rows of that segment (one contiguous row range)
  const long long q_begin = j0;
  long long next_end = seg_end;
  const long long tail_lo = seg_end - p.T;  // keys >= tail_lo are in the next segment's tail
  if ((pol & SEGATTN_TAIL) && seg_end == s0 + p.S && j_end > tail_lo && seg_end < N)
    next_end = seg_end + p.S < N ? seg_end + p.S : N;
  const int steps_per_head = (int)((next_end - q_begin + kBwdStep - 1) / kBwdStep);
  const int nsteps = steps_per_head * p.g;
  const long long q_stride = (long long)p.Hq * D;

  // per-lane bounds of the differentiable queries, as offsets from q_begin: rows [q_lo, q_lim).
  // Own segment: causal, i >= key.  Next segment: every row, if the key is in its carried tail.
  const long long jq = jw0 + col;
  const int q_lo = (int)(jq - q_begin);
  const int q_lim = jq < j_end ? (int)((jq >= tail_lo ? next_end : seg_end) - q_begin) : 0;

  // Wave-uniform bounds: a step whose 32 queries all lie in [q_lo_max, q_lim_min) needs no masks.
  const int q_lo_max = (int)(jw0 + 31 - q_begin);
  int q_lim_min = q_lim;
#pragma unroll
  for (int sh = 32; sh >= 1; sh >>= 1) q_lim_min = min(q_lim_min, __shfl_xor(q_lim_min, sh));
  q_lim_min = __builtin_amdgcn_readfirstlane(q_lim_min);

  // Fetch cursor: tiles are fetched in step order (query head major), one call per step; calls
  // beyond the last step repeat it (their data is never used).
  int f_head = 0, f_step = 0;
  const long long head0_q = ((b * N) * p.Hq + (long long)kv * p.g) * D;   // element offset of (b, row 0, first head)
  const long long head0_s = ((long long)b * p.Hq + (long long)kv * p.g) * N;
  int f_row[T::kLoads], f_col[T::kLoads];
#pragma unroll
  for (int i = 0; i < T::kLoads; ++i) {
    f_row[i] = (tid + 256 * i) / T::kChunks;
    f_col[i] = ((tid + 256 * i) % T::kChunks) * 8;
  }
  const int last_rel = (int)(next_end - 1 - q_begin);
  // (a macro rather than a lambda: register arrays handed to a lambda by reference end up in
  // scratch memory)
  u32x4 nq[T::kLoads], ng[T::kLoads];  // tile rows in flight: Q and dO (native vectors: they stay in registers)
  float ns = 0.f;                      // and this thread's row statistic
#define SEGATTN_BWD_FETCH_NEXT()                                                                      \
  do {                                                                                                \
    const int r0_ = f_step * kBwdStep;                                                                \
    const unsigned short *qb_ = a.q + head0_q + (long long)f_head * D + q_begin * q_stride;           \
    const unsigned short *gb_ = a.dout + head0_q + (long long)f_head * D + q_begin * q_stride;        \
    _Pragma("unroll") for (int i_ = 0; i_ < T::kLoads; ++i_) {                                        \
      int r_ = r0_ + f_row[i_];                                                                       \
      r_ = r_ < last_rel ? r_ : last_rel;                                                             \
      nq[i_] = *(const u32x4 *)(qb_ + (long long)r_ * q_stride + f_col[i_]);                          \
      ng[i_] = *(const u32x4 *)(gb_ + (long long)r_ * q_stride + f_col[i_]);                          \
    }                                                                                                 \
    if (tid < 2 * kBwdStep) {                                                                         \
      int r_ = r0_ + (tid & 31);                                                                      \
      r_ = r_ < last_rel ? r_ : last_rel;                                                             \
      const long long idx_ = head0_s + (long long)f_head * N + q_begin + r_;                          \
      ns = tid < kBwdStep ? a.lse[idx_] * kLog2e : a.delta[idx_];                                     \
    }                                                                                                 \
    if (!(f_head == p.g - 1 && f_step == steps_per_head - 1)) {                                       \
      f_step += 1;                                                                                    \
      if (f_step == steps_per_head) {                                                                 \
        f_step = 0;                                                                                   \
        f_head += 1;                                                                                  \
      }                                                                                               \
    }                                                                                                 \
  } while (0)
#define SEGATTN_BWD_STASH(buf)                                                                        \
  do {                                                                                                \
    _Pragma("unroll") for (int i_ = 0; i_ < T::kLoads; ++i_) {                                        \
      const int off_ = T::at(f_row[i_], f_col[i_] / 8);                                               \
      *(u32x4 *)(smem[buf][0] + off_) = nq[i_];                                                       \
      *(u32x4 *)(smem[buf][1] + off_) = ng[i_];                                                       \
    }                                                                                                 \
    if (tid < 2 * kBwdStep) stats[buf][tid >> 5][tid & 31] = ns;                                      \
  } while (0)

  // Software pipeline over the steps.  During step `it` the tile of step it+1 is written to the
  // other LDS buffer (fetched into registers one step earlier) and the tile of step it+2 is
  // fetched from HBM; one barrier in the middle of the step publishes tile it+1, after which the
  // row operands of step it+1 are read under the last products of step `it`.
  SEGATTN_BWD_FETCH_NEXT();
  SEGATTN_BWD_STASH(0);
  SEGATTN_BWD_FETCH_NEXT();
  __syncthreads();
  bf16x8 qa[NC], ga[NC];  // row operands of the current step
#pragma unroll
  for (int kc = 0; kc < NC; ++kc) {
    qa[kc] = read_row<D>(smem[0][0], lane, kc);
    ga[kc] = read_row<D>(smem[0][1], lane, kc);
  }
  int i_rel0 = 0;  // first query of the step, relative to q_begin
  for (int it = 0; it < nsteps; ++it) {
    const int cur = it & 1;
    const unsigned char *qt = smem[cur][0], *gt = smem[cur][1];
    SEGATTN_BWD_STASH(cur ^ 1);
    SEGATTN_BWD_FETCH_NEXT();
    __builtin_amdgcn_sched_barrier(0);
    // S, dP; behind them the transposed operands of the first 16 queries and the row statistics
    f32x16 S = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    f32x16 dP = S;
#pragma unroll
    for (int kc = 0; kc < NC; ++kc) {
      S = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qa[kc], Kr[kc], S, 0, 0, 0);
      dP = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ga[kc], Vr[kc], dP, 0, 0, 0);
    }
    bf16x8 gt0[NB], qt0[NB], gt1[NB], qt1[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      gt0[nb] = read_transposed<D>(gt, lane, nb, 0);
      qt0[nb] = read_transposed<D>(qt, lane, nb, 0);
    }
    f32x4 lse4[4], del4[4];  // row statistics of the lane's 16 query rows: rows 8 g + 4 hi .. +3
#pragma unroll
    for (int g4 = 0; g4 < 4; ++g4) {
      lse4[g4] = *(const f32x4 *)&stats[cur][0][8 * g4 + 4 * hi];
      del4[g4] = *(const f32x4 *)&stats[cur][1][8 * g4 + 4 * hi];
    }
    __builtin_amdgcn_sched_barrier(0);
    bf16x8 Pb[2], dSb[2];
    if (i_rel0 >= q_lo_max && i_rel0 + kBwdStep <= q_lim_min) {  // every pair of the tile counts
#pragma unroll
      for (int h2 = 0; h2 < 2; ++h2) {
        f32x8 e, f;
#pragma unroll
        for (int x = 0; x < 8; ++x) {
          const int r = 8 * h2 + x;
          const float pr = __builtin_amdgcn_exp2f(fmaf(S[r], c, -lse4[r / 4][r % 4]));
          e[x] = pr;
          f[x] = pr * (dP[r] - del4[r / 4][r % 4]);
        }
        Pb[h2] = __builtin_convertvector(e, bf16x8);
        dSb[h2] = __builtin_convertvector(f, bf16x8);
      }
    } else {
#pragma unroll
      for (int h2 = 0; h2 < 2; ++h2) {
        f32x8 e, f;
#pragma unroll
        for (int x = 0; x < 8; ++x) {
          const int r = 8 * h2 + x;
          const int rr = 8 * (r / 4) + 4 * hi + r % 4;  // query row inside the step
          const int i_rel = i_rel0 + rr;
          const bool ok = (i_rel >= q_lo) & (i_rel < q_lim);
          // a masked pair gets exponent -inf: its weight is exactly 0, without a branch
          const float pr = __builtin_amdgcn_exp2f(ok ? fmaf(S[r], c, -lse4[r / 4][r % 4]) : -INFINITY);
          e[x] = pr;
          f[x] = pr * (dP[r] - del4[r / 4][r % 4]);
        }
        Pb[h2] = __builtin_convertvector(e, bf16x8);
        dSb[h2] = __builtin_convertvector(f, bf16x8);
      }
    }
    i_rel0 += kBwdStep;
    if (i_rel0 >= steps_per_head * kBwdStep) i_rel0 = 0;
    __builtin_amdgcn_sched_barrier(0);
    // first 16 queries into dV^T, dK^T; behind them the transposed operands of the other 16
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      gt1[nb] = read_transposed<D>(gt, lane, nb, 1);
      qt1[nb] = read_transposed<D>(qt, lane, nb, 1);
    }
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      mma_acc(dVa[nb], gt0[nb], Pb[0]);
      mma_acc(dKa[nb], qt0[nb], dSb[0]);
    }
    __builtin_amdgcn_sched_barrier(0);
    __syncthreads();  // tile it+1 is in LDS for everyone; nobody reads tile `it` any more
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int kc = 0; kc < NC; ++kc) {
      qa[kc] = read_row<D>(smem[cur ^ 1][0], lane, kc);
      ga[kc] = read_row<D>(smem[cur ^ 1][1], lane, kc);
    }
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      mma_acc(dVa[nb], gt1[nb], Pb[1]);
      mma_acc(dKa[nb], qt1[nb], dSb[1]);
    }
    __builtin_amdgcn_sched_barrier(0);
  }
#undef SEGATTN_BWD_FETCH_NEXT
#undef SEGATTN_BWD_STASH
  if (!key_ok) return;
#pragma unroll
  for (int nb = 0; nb < NB; ++nb)
#pragma unroll
    for (int rg = 0; rg < 4; ++rg) {
      const int d = 32 * nb + 8 * rg + 4 * hi;
      const f32x4 gk = {dKa[nb][4 * rg + 0] * p.scale, dKa[nb][4 * rg + 1] * p.scale,
                        dKa[nb][4 * rg + 2] * p.scale, dKa[nb][4 * rg + 3] * p.scale};
      const f32x4 gv = {dVa[nb][4 * rg + 0], dVa[nb][4 * rg + 1], dVa[nb][4 * rg + 2],
                        dVa[nb][4 * rg + 3]};
      if (p.out_fp32) {
        *(f32x4 *)((float *)a.dk + koff + d) = gk;
        *(f32x4 *)((float *)a.dv + koff + d) = gv;
      } else {
        *(uint2 *)((unsigned short *)a.dk + koff + d) = __builtin_bit_cast(uint2, __builtin_convertvector(gk, bf16x4));
        *(uint2 *)((unsigned short *)a.dv + koff + d) = __builtin_bit_cast(uint2, __builtin_convertvector(gv, bf16x4));
      }
    }
}

// ---------------------------------------------------------------------------------------------
// launch
// ---------------------------------------------------------------------------------------------
static int bwd_heads_per_wg(const Problem &p) { return (p.g % 4 == 0) ? 4 : (p.g % 2 == 0) ? 2 : 1; }

template <int D>
static hipError_t launch_bwd_d(const Problem &p, const BwdArgs &a, hipStream_t st) {
  const int hs = bwd_heads_per_wg(p);
  const int rows = (4 / hs) * 32;
  PrefillArgs pa;
  memset(&pa, 0, sizeof(pa));
  pa.q = a.q;
  pa.k = a.k;
  pa.v = a.v;
  pa.out = a.dq;
  pa.lse = const_cast<float *>(a.lse);
  pa.cache = nullptr;
  pa.n_rows = a.n;
  pa.n_seg = (a.n + p.S - 1) / p.S;
  const long long seg_rows = a.n < p.S ? a.n : p.S;
  pa.q_blocks_per_seg = (int)((seg_rows + rows - 1) / rows);
  pa.pair_stride = prefill_pair_stride((long long)p.B * (p.Hkv - p.n_past) * (p.g / hs) * pa.n_seg);
  const long long grid_q = (long long)p.B * p.Hkv * (p.g / hs) * pa.n_seg * pa.q_blocks_per_seg;
  const int blocks_per_seg = (int)((seg_rows + 127) / 128);
  const long long grid_k = (long long)p.B * p.Hkv * pa.n_seg * blocks_per_seg;
  if (grid_q <= 0 || grid_q > 0x7fffffffLL || grid_k > 0x7fffffffLL) return hipErrorInvalidValue;
  if (hs == 4) hipLaunchKernelGGL((bwd_dq_kernel<D, 4>), dim3((unsigned)grid_q), dim3(256), 0, st, p, pa, a);
  else if (hs == 2) hipLaunchKernelGGL((bwd_dq_kernel<D, 2>), dim3((unsigned)grid_q), dim3(256), 0, st, p, pa, a);
  else hipLaunchKernelGGL((bwd_dq_kernel<D, 1>), dim3((unsigned)grid_q), dim3(256), 0, st, p, pa, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(bwd_dkv_kernel<D>, dim3((unsigned)grid_k), dim3(256), 0, st, p, a, blocks_per_seg, pa.n_seg);
  return hipGetLastError();
}

hipError_t launch_bwd_mfma(const Problem &p, const BwdArgs &a, hipStream_t st) {
  return p.D == 128 ? launch_bwd_d<128>(p, a, st) : launch_bwd_d<64>(p, a, st);
}

}  // namespace segattn
