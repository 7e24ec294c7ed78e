// dQ kernel of the bf16 MFMA backward of segment-level attention (see segattn_bwd_mfma.hip for
// the scheme).  A wave owns 32 query rows of one head and walks the keys it sees in steps of 32
// (prefix span, then its own segment up to the diagonal):
//   S^T  = K . Q^T          P^T = exp2(S^T c - LSE)
//   dP^T = V . dO^T         dS^T = P^T (dP^T - delta)
//   dQ^T += K^T . dS^T      (every visible key contributes, past rows too)
// Built with the compiler's VGPR form of the matrix products (-amdgpu-mfma-vgpr-form): the whole
// state of a wave -- Q^T and dO^T operands, the dQ^T accumulators, the score tiles -- fits 256
// vector registers, so two workgroups share a CU and one fills the other's stalls (each step is
// a chain products -> exponentials -> products with a barrier at its end).
#include <string.h>

#include "segattn_bwd_tiles.h"

namespace segattn {

// ---------------------------------------------------------------------------------------------
// dQ
// ---------------------------------------------------------------------------------------------
// One work item (query block x head sub-group): see bwd_dq_kernel for how items reach workgroups.
// next_from: nullptr, or the queue counter the workgroup takes its next item from; thread 0 draws
// the ticket after the last K/V step and hands it back (other threads: 0).
template <int D, int HS>
__device__ __forceinline__ unsigned bwd_dq_item(const Problem &p, const PrefillArgs &pa, const BwdArgs &a,
                                                const int bid, unsigned char (&smem)[2][2][BwdTile<D>::kBytes],
                                                unsigned *const next_from) {
  using T = BwdTile<D>;
  constexpr int NC = D / 16, NB = D / 32;
  constexpr int RW = 32;             // query rows per wave
  constexpr int BQ = (4 / HS) * RW;  // query rows per workgroup

  WorkItem w = resolve(p, pa, bid, BQ, HS);
  if (!w.valid) return (next_from && threadIdx.x == 0) ? atomicAdd(next_from, 1u) : 0u;
  pin_uniform(w);
  int tid = threadIdx.x;
  asm volatile("" : "+v"(tid));  // not a loop invariant of the caller's loop (see prefill_mfma_kernel)
  const int wave = tid >> 6, lane = tid & 63;
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
  const long long stat = (w.lse - a.lse) + (long long)head * w.lse_head_stride + t;  // index into lse / delta
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

  // Tiles of step j (clamped to the last step, whose re-fetch is not used): global -> registers.
  // A scalar base per step plus a 32-bit lane offset fixed for the kernel (both spans have the
  // same row stride here: the backward pass reads K/V by absolute position); only the last step
  // of a span can reach past its end, and only then are the lane's rows clamped.
  const unsigned row_bytes = (unsigned)(w.stride1 * 2);
  int f_row[T::kLoads];
  unsigned f_col2[T::kLoads], f_off[T::kLoads];
#pragma unroll
  for (int i = 0; i < T::kLoads; ++i) {
    f_row[i] = (tid + 256 * i) / T::kChunks;
    f_col2[i] = (unsigned)((tid + 256 * i) % T::kChunks) * 16;
    f_off[i] = (unsigned)f_row[i] * row_bytes + f_col2[i];
  }
  u32x4 kr[T::kLoads], vr[T::kLoads];
#define SEGATTN_BWD_FETCH_KV(jj)                                                                      \
  do {                                                                                                \
    int j_ = (jj);                                                                                    \
    j_ = j_ < nsteps ? j_ : nsteps - 1;                                                               \
    const bool s1_ = j_ >= nst0;                                                                      \
    const int jl_ = s1_ ? j_ - nst0 : j_;                                                             \
    const int left_ = (s1_ ? w.n1 : w.n0) - jl_ * kBwdStep;                                           \
    const unsigned long long so_ = (unsigned long long)jl_ * kBwdStep * row_bytes;                    \
    const GLB_AS unsigned char *kb_ = (const GLB_AS unsigned char *)(s1_ ? w.k1 : w.k0) + so_;        \
    const GLB_AS unsigned char *vb_ = (const GLB_AS unsigned char *)(s1_ ? w.v1 : w.v0) + so_;        \
    if (left_ >= kBwdStep) {                                                                          \
      _Pragma("unroll") for (int i_ = 0; i_ < T::kLoads; ++i_) {                                      \
        kr[i_] = *(const GLB_AS u32x4 *)(kb_ + f_off[i_]);                                            \
        vr[i_] = *(const GLB_AS u32x4 *)(vb_ + f_off[i_]);                                            \
      }                                                                                               \
    } else {                                                                                          \
      _Pragma("unroll") for (int i_ = 0; i_ < T::kLoads; ++i_) {                                      \
        const int r_ = f_row[i_] < left_ ? f_row[i_] : left_ - 1;                                     \
        const unsigned o_ = (unsigned)r_ * row_bytes + f_col2[i_];                                    \
        kr[i_] = *(const GLB_AS u32x4 *)(kb_ + o_);                                                   \
        vr[i_] = *(const GLB_AS u32x4 *)(vb_ + o_);                                                   \
      }                                                                                               \
    }                                                                                                 \
  } while (0)
#define SEGATTN_BWD_STORE_KV(buf)                                                                     \
  do {                                                                                                \
    _Pragma("unroll") for (int i_ = 0; i_ < T::kLoads; ++i_) {                                        \
      const int off_ = T::at(f_row[i_], (int)(f_col2[i_] / 16));                                      \
      *(u32x4 *)(smem[buf][0] + off_) = kr[i_];                                                       \
      *(u32x4 *)(smem[buf][1] + off_) = vr[i_];                                                       \
    }                                                                                                 \
  } while (0)
  SEGATTN_BWD_FETCH_KV(0);
  SEGATTN_BWD_STORE_KV(0);
  __syncthreads();
  (void)my_last;
  for (int j = 0; j < nsteps; ++j) {
    const int cur = j & 1;
    SEGATTN_BWD_FETCH_KV(j + 1);
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
      // a step whose 32 keys are visible to all 32 queries of the wave needs no masks: keys of the
      // prefix span short of its ragged end, keys of the own segment up to the wave's first row
      const bool all_visible = own ? (k0 + kBwdStep - 1 <= tw0 && tw0 + RW - 1 <= last_row) : (k0 + kBwdStep <= span_len);
      if (all_visible) {
#pragma unroll
        for (int h2 = 0; h2 < 2; ++h2) {
          f32x8 e;
#pragma unroll
          for (int x = 0; x < 8; ++x) {
            const int r = 8 * h2 + x;
            e[x] = __builtin_amdgcn_exp2f(fmaf(S[r], c, -lse2)) * (dP[r] - delta);
          }
          dS[h2] = __builtin_convertvector(e, bf16x8);
        }
      } else {
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
      }
#pragma unroll
      for (int h2 = 0; h2 < 2; ++h2)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) mma_acc(acc[nb], read_transposed<D>(kt, lane, nb, h2), dS[h2]);
    }
    SEGATTN_BWD_STORE_KV(cur ^ 1);
    __syncthreads();
  }
#undef SEGATTN_BWD_FETCH_KV
#undef SEGATTN_BWD_STORE_KV
  unsigned ticket = 0;
  if (next_from && tid == 0) ticket = atomicAdd(next_from, 1u);
  if (row_ok) {
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
  return ticket;
}

// One item per workgroup (pa.queue == nullptr), or a resident grid that takes item after item from
// the per-XCD queues, as the forward kernel does and for the same reasons (prefill_mfma_kernel).
template <int D, int HS>
__global__ __launch_bounds__(256, 2) void bwd_dq_kernel(const Problem p_arg, const PrefillArgs pa_arg, const BwdArgs a_arg) {
  __shared__ __attribute__((aligned(16))) unsigned char smem[2][2][BwdTile<D>::kBytes];  // [buffer][K,V]
  __shared__ int claim;
  constexpr unsigned kPaAt = (sizeof(Problem) + alignof(PrefillArgs) - 1) / alignof(PrefillArgs) * alignof(PrefillArgs);
  constexpr unsigned kAAt = (kPaAt + sizeof(PrefillArgs) + alignof(BwdArgs) - 1) / alignof(BwdArgs) * alignof(BwdArgs);
  unsigned ticket = 0;
  bool drawn = false;
  for (;;) {
    // arguments through an opaque pointer, once per round: see prefill_mfma_kernel
    const __attribute__((address_space(4))) unsigned char *ka =
        (const __attribute__((address_space(4))) unsigned char *)__builtin_amdgcn_kernarg_segment_ptr();
    asm volatile("" : "+s"(ka));
    const Problem &p = *(const Problem *)ka;
    const PrefillArgs &pa = *(const PrefillArgs *)(ka + kPaAt);
    const BwdArgs &a = *(const BwdArgs *)(ka + kAAt);
    int bid = (int)blockIdx.x;
    const bool queued = pa.queue != nullptr;
    unsigned *const own = queued ? pa.queue + kQueueStride * ((int)blockIdx.x & 7) : nullptr;
    if (queued) {
      bid = take_item(pa.queue, pa.grid_items, drawn, ticket, &claim);
      if (bid < 0) return;
    }
    ticket = bwd_dq_item<D, HS>(p, pa, a, bid, smem, own);
    drawn = true;
    if (!queued) return;
    __syncthreads();  // the item's last reads of the tiles come before the next item's first stores
  }
}

static int bwd_heads_per_wg(const Problem &p) { return (p.g % 4 == 0) ? 4 : (p.g % 2 == 0) ? 2 : 1; }

template <int D>
static hipError_t launch_dq(const Problem &p, const BwdArgs &a, hipStream_t st) {
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
  pa.cu_seqlens = a.cu_seqlens;
  pa.total_rows = a.total;
  pa.n_seg = (a.n + p.S - 1) / p.S;
  const long long seg_rows = a.n < p.S ? a.n : p.S;
  pa.q_blocks_per_seg = (int)((seg_rows + rows - 1) / rows);
  pa.pair_stride = prefill_pair_stride((long long)p.B * (p.Hkv - p.n_past) * (p.g / hs) * pa.n_seg);
  const long long grid_q = (long long)p.B * p.Hkv * (p.g / hs) * pa.n_seg * pa.q_blocks_per_seg;
  if (grid_q <= 0 || grid_q > 0x7fffffffLL) return hipErrorInvalidValue;
  pa.grid_items = (int)grid_q;
  // resident grid + item queues where every resident workgroup would get more than two items
  const void *kern = hs == 4 ? (const void *)bwd_dq_kernel<D, 4> : hs == 2 ? (const void *)bwd_dq_kernel<D, 2>
                                                                            : (const void *)bwd_dq_kernel<D, 1>;
  static ResidentCount resident_count[3];  // per heads-per-workgroup instantiation, asked once
  const int resident = p.tune_queue == 1 ? 0 : resident_count[hs == 4 ? 2 : hs == 2 ? 1 : 0].get(kern, 256, 0);
  long long launch = item_queue_grid(p, grid_q, resident);
  if (launch != grid_q || (p.tune_queue >= 2 && grid_q > 1 && resident > 0)) {
    pa.queue = item_queue_for(st);
    if (!pa.queue) launch = grid_q;
  }
  std::unique_lock<std::mutex> pair;  // reset and launch enter the stream back to back
  if (pa.queue) {
    pair = std::unique_lock<std::mutex>(item_queue_launch_mutex());
    hipError_t e = item_queue_reset(pa.queue, st);
    if (e != hipSuccess) return e;
  }
  if (hs == 4) hipLaunchKernelGGL((bwd_dq_kernel<D, 4>), dim3((unsigned)launch), dim3(256), 0, st, p, pa, a);
  else if (hs == 2) hipLaunchKernelGGL((bwd_dq_kernel<D, 2>), dim3((unsigned)launch), dim3(256), 0, st, p, pa, a);
  else hipLaunchKernelGGL((bwd_dq_kernel<D, 1>), dim3((unsigned)launch), dim3(256), 0, st, p, pa, a);
  return hipGetLastError();
}

hipError_t launch_bwd_dq(const Problem &p, const BwdArgs &a, hipStream_t st) {
  return p.D == 128 ? launch_dq<128>(p, a, st) : launch_dq<64>(p, a, st);
}

}  // namespace segattn
