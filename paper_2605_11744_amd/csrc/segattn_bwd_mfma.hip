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
// This file and segattn_bwd_dq.hip are compiled with the VGPR form of the matrix products
// (-amdgpu-mfma-vgpr-form): S and dP arrive in vector registers, where the exponentials read them.
// In the dK/dV kernel the K and V operands sit in accumulation registers (park()), which a product
// reads directly; with the default form the compiler also kept S and dP there and moved two
// accumulator blocks back and forth every step to make room (96 register moves per 32 products).
// All products are builtins, so the compiler tracks every MFMA hazard itself.
#include <string.h>

#include "segattn_bwd_tiles.h"

namespace segattn {

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

  // blockIdx -> (key block, segment, kv head, b), longest work first: the key blocks that reach
  // into the carried tail come first (they also see the whole next segment), then the others from
  // the start of the segment on.  The (segment, head, sequence) of a workgroup rotates with the
  // block index: workgroups go to the XCDs round-robin in index order, and with a fixed assignment
  // an XCD would see one segment only -- the last segment's blocks have no next segment and are a
  // third shorter, so half of the XCDs would wait for the other half.
  const int per = n_seg * p.Hkv * p.B;
  const int ord = blockIdx.x / per;
  const int kb_tail = (int)((p.S - p.T) / BK);  // first key block with keys in the tail
  const int n_tail = p.T > 0 && kb_tail < blocks_per_seg ? blocks_per_seg - kb_tail : 0;
  const int kb = ord < n_tail ? kb_tail + ord : ord - n_tail;
  int rest = (blockIdx.x % per + ord) % per;
  const int seg = rest % n_seg;
  rest /= n_seg;
  const int kv = rest % p.Hkv;
  const int b = rest / p.Hkv;
  const int pol = p.policy[kv];
  SeqSpan sq = seq_span(p, a, b);  // the same for the whole workgroup: keep it in scalar registers
  sq.row0 = uniform_i64(sq.row0);
  sq.n = uniform_i64(sq.n);
  sq.stat0 = uniform_i64(sq.stat0);
  sq.stat_stride = uniform_i64(sq.stat_stride);
  const long long N = sq.n;
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
  const long long koff = ((sq.row0 + jk) * p.Hkv + kv) * D;
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
  // beyond the last step repeat it (their data is never used).  Addresses are a scalar base that
  // moves with the cursor plus a 32-bit lane offset fixed for the whole kernel; only the last step
  // of a head can reach past the last query row, and only then are the lane's rows clamped.
  int f_head = 0, f_step = 0;
  const long long head0_q = (sq.row0 * p.Hq + (long long)kv * p.g) * D;   // element offset of (b, row 0, first head)
  const long long head0_s = sq.stat0 + (long long)kv * p.g * sq.stat_stride;
  const unsigned char *fq0 = (const unsigned char *)(a.q + head0_q + q_begin * q_stride);
  const unsigned char *fg0 = (const unsigned char *)(a.dout + head0_q + q_begin * q_stride);
  const unsigned row_bytes = (unsigned)(q_stride * 2);
  int f_row[T::kLoads], f_col[T::kLoads];
  unsigned f_off[T::kLoads];  // byte offset of the lane's chunk inside a 32-row tile of one head
#pragma unroll
  for (int i = 0; i < T::kLoads; ++i) {
    f_row[i] = (tid + 256 * i) / T::kChunks;
    f_col[i] = ((tid + 256 * i) % T::kChunks) * 8;
    f_off[i] = (unsigned)f_row[i] * row_bytes + (unsigned)f_col[i] * 2;
  }
  const int last_rel = (int)(next_end - 1 - q_begin);
  // the lane's row statistic: lanes 0..31 of the first wave fetch LSE, lanes 32..63 delta
  const float *f_stat0 = (tid < kBwdStep ? a.lse : a.delta) + head0_s + q_begin;
  // (a macro rather than a lambda: register arrays handed to a lambda by reference end up in
  // scratch memory)
  u32x4 nq[T::kLoads], ng[T::kLoads];  // tile rows in flight: Q and dO (native vectors: they stay in registers)
  float ns = 0.f;                      // and this thread's row statistic, as stored (LSE is scaled when stashed,
                                       // so that nothing waits for the load inside the step that issues it)
#define SEGATTN_BWD_FETCH_NEXT()                                                                      \
  do {                                                                                                \
    const int r0_ = f_step * kBwdStep;                                                                \
    const unsigned long long so_ = (unsigned long long)f_head * (D * 2) + (unsigned long long)r0_ * row_bytes; \
    const unsigned char *qb_ = fq0 + so_, *gb_ = fg0 + so_;                                           \
    if (r0_ + kBwdStep - 1 <= last_rel) {                                                             \
      _Pragma("unroll") for (int i_ = 0; i_ < T::kLoads; ++i_) {                                      \
        nq[i_] = *(const u32x4 *)(qb_ + f_off[i_]);                                                   \
        ng[i_] = *(const u32x4 *)(gb_ + f_off[i_]);                                                   \
      }                                                                                               \
    } else {                                                                                          \
      _Pragma("unroll") for (int i_ = 0; i_ < T::kLoads; ++i_) {                                      \
        const int r_ = r0_ + f_row[i_] < last_rel ? f_row[i_] : last_rel - r0_;                      \
        const unsigned o_ = (unsigned)r_ * row_bytes + (unsigned)f_col[i_] * 2;                       \
        nq[i_] = *(const u32x4 *)(qb_ + o_);                                                          \
        ng[i_] = *(const u32x4 *)(gb_ + o_);                                                          \
      }                                                                                               \
    }                                                                                                 \
    if (tid < 2 * kBwdStep) {                                                                         \
      int r_ = r0_ + (tid & 31);                                                                      \
      r_ = r_ < last_rel ? r_ : last_rel;                                                             \
      ns = f_stat0[(long long)f_head * sq.stat_stride + r_];                                          \
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
    if (tid < 2 * kBwdStep) stats[buf][tid >> 5][tid & 31] = tid < kBwdStep ? ns * kLog2e : ns;           \
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
template <int D>
static hipError_t launch_dkv(const Problem &p, const BwdArgs &a, hipStream_t st) {
  const int n_seg = (a.n + p.S - 1) / p.S;
  const long long seg_rows = a.n < p.S ? a.n : p.S;
  const int blocks_per_seg = (int)((seg_rows + 127) / 128);
  const long long grid_k = (long long)p.B * p.Hkv * n_seg * blocks_per_seg;
  if (grid_k <= 0 || grid_k > 0x7fffffffLL) return hipErrorInvalidValue;
  hipLaunchKernelGGL(bwd_dkv_kernel<D>, dim3((unsigned)grid_k), dim3(256), 0, st, p, a, blocks_per_seg, n_seg);
  return hipGetLastError();
}

hipError_t launch_bwd_mfma(const Problem &p, const BwdArgs &a, hipStream_t st) {
  const hipError_t e = launch_bwd_dq(p, a, st);
  if (e != hipSuccess) return e;
  return p.D == 128 ? launch_dkv<128>(p, a, st) : launch_dkv<64>(p, a, st);
}

}  // namespace segattn
