// dQ kernel of the bf16 MFMA backward of segment-level attention (see segattn_bwd_mfma.hip for
// the scheme).  A wave owns 32 query rows of one head and walks the keys it sees in steps of 32
// (prefix span, then its own segment up to the diagonal):
//   S^T  = K . Q^T          P^T = exp2(S^T c - LSE)
//   dP^T = V . dO^T         dS^T = P^T (dP^T - delta)
//   dQ^T += K^T . dS^T      (every visible key contributes, past rows too)
// K/V tiles travel HBM -> LDS by DMA into a ring of three step buffers, two steps ahead of their
// use; one barrier per step.  Built with the compiler's VGPR form of the matrix products (-amdgpu-mfma-vgpr-form): the whole
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
// LDS of the dQ kernel: a ring of three step buffers, [K tile][V tile] each.
template <int D>
struct DqGeom {
  static constexpr int kTile = BwdTile<D>::kBytes;
  static constexpr int kBuf = 2 * kTile;
  static constexpr int kBufs = 3;
  static constexpr int kBytes = kBufs * kBuf;
};

template <int D, int HS>
__device__ __forceinline__ unsigned bwd_dq_item(const Problem &p, const PrefillArgs &pa, const BwdArgs &a,
                                                const int bid, unsigned char *const smem, unsigned *const next_from) {
  using T = BwdTile<D>;
  using G = DqGeom<D>;
  constexpr int NC = D / 16, NB = D / 32;
  constexpr int RW = 32;             // query rows per wave
  constexpr int BQ = (4 / HS) * RW;  // query rows per workgroup
  constexpr int kTile = G::kTile, kBuf = G::kBuf, NBUF = G::kBufs;
  constexpr int LPW = T::kChunks / 8;     // wave-wide 1 KB loads per tensor, step and wave
  constexpr int kLoadsPerStep = 2 * LPW;  // per wave: K, V
  static_assert((NBUF - 1) * kBuf + kTile + 16 * T::kRowBytes < 65536, "LDS offsets must fit the 16-bit immediate");

  WorkItem w = resolve(p, pa, bid, BQ, HS);
  if (!w.valid) return (next_from && threadIdx.x == 0) ? atomicAdd(next_from, 1u) : 0u;
  pin_uniform(w);
  int tid = threadIdx.x;
  asm volatile("" : "+v"(tid));  // not a loop invariant of the caller's loop (see prefill_mfma_kernel)
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int hi = lane >> 5, col = lane & 31, i16 = lane & 15, g16 = (lane >> 4) & 1;
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
  const long long stat = (w.lse - a.lse) + (long long)head * w.lse_head_stride + t;  // index into the row statistics
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

  // ---- HBM -> LDS by DMA (global_load_lds): load i of a wave covers bytes [(wave LPW + i) 1024,
  // +1024) of a tile, i.e. row (wave LPW + i) rows-per-KB + lane / chunks, chunk slot lane % chunks,
  // which receives the global chunk slot ^ swz(row): the tile's swizzle applied on the global side
  // (the LDS side of such a load is linear in the lane).  Both spans have the same row stride here
  // (the backward pass reads K/V by absolute position).  The fetch cursor walks the steps in
  // order and stays on the last one (fetched again, never read), so every wait is one constant.
  const unsigned row_bytes = (unsigned)(w.stride1 * 2);
  constexpr int kRowsPerKB = 1024 / T::kRowBytes;
  int f_row[LPW];
  unsigned f_chunk[LPW], f_off[LPW];
#pragma unroll
  for (int i = 0; i < LPW; ++i) {
    f_row[i] = (wave * LPW + i) * kRowsPerKB + lane / T::kChunks;
    f_chunk[i] = (unsigned)(((lane % T::kChunks) ^ T::swz(f_row[i])) << 4);
    f_off[i] = (unsigned)f_row[i] * row_bytes + f_chunk[i];
  }
  LDS_AS unsigned char *const lds = (LDS_AS unsigned char *)smem;
  const unsigned lds_base = (unsigned)(size_t)lds;
  int f_j = 0, f_left = nst0 > 0 ? w.n0 : w.n1;  // step to fetch next, rows its span has from its first row on
  const unsigned char *f_k = (const unsigned char *)(nst0 > 0 ? w.k0 : w.k1);
  const unsigned char *f_v = (const unsigned char *)(nst0 > 0 ? w.v0 : w.v1);
  auto fetch_next = [&](int buf) __attribute__((always_inline)) {
    LDS_AS unsigned char *dst = lds + buf * kBuf + wave * (LPW * 1024);
    if (f_left >= kBwdStep) {
#pragma unroll
      for (int i = 0; i < LPW; ++i) {
        // (through an empty asm, so that the lane offset is widened to 64 bits here, next to the
        // addition: the load then takes a scalar base plus a 32-bit lane offset)
        asm volatile("" : "+v"(f_off[i]));
        __builtin_amdgcn_global_load_lds((const GLB_AS void *)(f_k + f_off[i]), (LDS_AS void *)(dst + i * 1024), 16, 0, 0);
        __builtin_amdgcn_global_load_lds((const GLB_AS void *)(f_v + f_off[i]), (LDS_AS void *)(dst + kTile + i * 1024), 16, 0, 0);
      }
    } else {  // the last step of a span can reach past its end: clamp the lane's rows
#pragma unroll
      for (int i = 0; i < LPW; ++i) {
        const int r = f_row[i] < f_left ? f_row[i] : f_left - 1;
        const unsigned o = (unsigned)r * row_bytes + f_chunk[i];
        __builtin_amdgcn_global_load_lds((const GLB_AS void *)(f_k + o), (LDS_AS void *)(dst + i * 1024), 16, 0, 0);
        __builtin_amdgcn_global_load_lds((const GLB_AS void *)(f_v + o), (LDS_AS void *)(dst + kTile + i * 1024), 16, 0, 0);
      }
    }
    if (f_j + 1 < nsteps) {
      f_j += 1;
      if (f_j == nst0) {  // on to the own segment
        f_k = (const unsigned char *)w.k1;
        f_v = (const unsigned char *)w.v1;
        f_left = w.n1;
      } else {
        f_k += (size_t)kBwdStep * row_bytes;
        f_v += (size_t)kBwdStep * row_bytes;
        f_left -= kBwdStep;
      }
    }
  };
#define SEGATTN_VMCNT(N) __builtin_amdgcn_s_waitcnt(0x0F70 | ((N) & 15) | (((N) >> 4) << 14))

  // ---- per-lane LDS read addresses inside a step buffer (buffer and tensor are immediates)
  unsigned ro[NC];  // row operands: tile row `col`, logical chunk 2 kc + hi
#pragma unroll
  for (int kc = 0; kc < NC; ++kc) ro[kc] = lds_base + (unsigned)T::at(col, 2 * kc + hi);
  unsigned tro[NB][2];  // transposed operands (see read_transposed); rows 16 apart share the swizzle: h2 is an immediate
#pragma unroll
  for (int nb = 0; nb < NB; ++nb)
#pragma unroll
    for (int u = 0; u < 2; ++u)
      tro[nb][u] = lds_base + (unsigned)(T::at(4 * hi + (i16 >> 2) + 8 * u, 4 * nb + 2 * g16 + ((i16 & 3) >> 1)) + 8 * (i16 & 1));
  static_assert(T::swz(0) == T::swz(16) && T::swz(5) == T::swz(21) && T::swz(15) == T::swz(31), "h2 as an immediate");
  typedef int i32x4 __attribute__((ext_vector_type(4)));

  // One step on the tile in buffer B (LDS reads are inline asm with explicit waits: the compiler
  // would make every LDS read wait for all outstanding DMA):
  //   request the tile two steps on (its buffer was last read before the previous barrier)
  //   S^T = K Q^T, dP^T = V dO^T (row operands from LDS, in two halves), with the transposed K
  //   operands read behind the second half's products
  //   dS^T = exp2(S^T c - LSE) (dP^T - delta) (keys the queries may not see get score -inf first), bf16
  //   dQ^T += K^T dS^T
  //   the next step's tile has landed (this wave's part); barrier: everyone's, and nobody reads
  //   this step's tile any more
#define SEGATTN_DQ_STEP(B)                                                                                       \
  do {                                                                                                           \
    constexpr int BO = (B) * kBuf, BF = ((B) + NBUF - 1) % NBUF;                                                 \
    const bool own = j >= nst0;                                                                                  \
    const int k0 = (own ? j - nst0 : j) * kBwdStep; /* first key of the step inside its span */                  \
    const int span_len = own ? w.n1 : w.n0;                                                                      \
    /* a step whose 32 keys are visible to all 32 queries of the wave needs no masks: keys of the prefix         \
       span short of its ragged end, keys of the own segment up to the wave's first row */                       \
    const bool all_visible = own ? (k0 + kBwdStep - 1 <= tw0 && tw0 + RW - 1 <= last_row) : (k0 + kBwdStep <= span_len); \
    fetch_next(BF);                                                                                              \
    __builtin_amdgcn_sched_barrier(0);                                                                           \
    /* row operands in two halves (registers: the second half takes the place of the first as its products     \
       are issued); the transposed K operands are read behind the second half's products */                      \
    i32x4 ka[NC], va[NC];                                                                                        \
    s16x4 kt[2][NB][2];                                                                                          \
    _Pragma("unroll") for (int kc = 0; kc < NC / 2; ++kc) {                                                      \
      asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(ka[kc]) : "v"(ro[kc]), "n"(BO));                       \
      asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(va[kc]) : "v"(ro[kc]), "n"(BO + kTile));               \
    }                                                                                                            \
    SEGATTN_DQ_ROWS_WAIT(0);                                                                                     \
    f32x16 S = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};                 \
    f32x16 dP = S;                                                                                               \
    __builtin_amdgcn_sched_barrier(0);                                                                           \
    _Pragma("unroll") for (int kc = 0; kc < NC / 2; ++kc) {                                                      \
      S = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, ka[kc]), Qr[kc], S, 0, 0, 0);       \
      dP = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, va[kc]), Gr[kc], dP, 0, 0, 0);     \
      __builtin_amdgcn_sched_barrier(0);                                                                         \
      asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(ka[kc + NC / 2]) : "v"(ro[kc + NC / 2]), "n"(BO));     \
      asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(va[kc + NC / 2]) : "v"(ro[kc + NC / 2]), "n"(BO + kTile)); \
      __builtin_amdgcn_sched_barrier(0);                                                                         \
    }                                                                                                            \
    SEGATTN_DQ_ROWS_WAIT(NC / 2);                                                                                \
    __builtin_amdgcn_sched_barrier(0);                                                                           \
    _Pragma("unroll") for (int kc = NC / 2; kc < NC; ++kc) {                                                     \
      S = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, ka[kc]), Qr[kc], S, 0, 0, 0);       \
      dP = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, va[kc]), Gr[kc], dP, 0, 0, 0);     \
      __builtin_amdgcn_sched_barrier(0);                                                                         \
      { /* 4 NB transposed reads over NC / 2 product pairs */                                                    \
        constexpr int per = 4 * NB / (NC / 2);                                                                   \
        _Pragma("unroll") for (int e = 0; e < per; ++e) {                                                        \
          const int idx = (kc - NC / 2) * per + e, h2 = idx / (2 * NB), nb = (idx / 2) % NB, u = idx % 2;        \
          if (h2 == 0)                                                                                           \
            asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(kt[0][nb][u]) : "v"(tro[nb][u]), "n"(BO));  \
          else                                                                                                   \
            asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(kt[1][nb][u]) : "v"(tro[nb][u]), "n"(BO + 16 * T::kRowBytes)); \
        }                                                                                                        \
      }                                                                                                          \
      __builtin_amdgcn_sched_barrier(0);                                                                         \
    }                                                                                                            \
    if (__builtin_expect(!all_visible, 0)) { /* rare: laid out off the step's straight path */                   \
      const int kmax = own ? (t < span_len - 1 ? t : span_len - 1) : span_len - 1; /* last visible key of the span */ \
      _Pragma("unroll") for (int r = 0; r < 16; ++r)                                                             \
        S[r] = (k0 + 8 * (r / 4) + 4 * hi + r % 4 <= kmax) ? S[r] : -INFINITY; /* weight exactly 0 */            \
    }                                                                                                            \
    bf16x8 dS[2];                                                                                                \
    _Pragma("unroll") for (int h2 = 0; h2 < 2; ++h2) {                                                           \
      f32x8 e;                                                                                                   \
      _Pragma("unroll") for (int x = 0; x < 8; ++x)                                                              \
        e[x] = __builtin_amdgcn_exp2f(fmaf(S[8 * h2 + x], c, -lse2)) * (dP[8 * h2 + x] - delta);                 \
      dS[h2] = __builtin_convertvector(e, bf16x8);                                                               \
    }                                                                                                            \
    SEGATTN_DQ_TR_WAIT();                                                                                        \
    __builtin_amdgcn_sched_barrier(0);                                                                           \
    _Pragma("unroll") for (int h2 = 0; h2 < 2; ++h2)                                                             \
      _Pragma("unroll") for (int nb = 0; nb < NB; ++nb)                                                          \
        mma_acc(acc[nb], __builtin_bit_cast(bf16x8, __builtin_shufflevector(kt[h2][nb][0], kt[h2][nb][1], 0, 1, 2, 3, 4, 5, 6, 7)), dS[h2]); \
    __builtin_amdgcn_sched_barrier(0);                                                                           \
    SEGATTN_VMCNT(kLoadsPerStep);                                                                                \
    __builtin_amdgcn_s_barrier();                                                                                \
    __builtin_amdgcn_sched_barrier(0);                                                                           \
  } while (0)
#define SEGATTN_DQ_ROWS_WAIT(F) /* the NC / 2 row operand pairs from index F on have arrived */                \
  do {                                                                                                           \
    if constexpr (NC == 8) {                                                                                     \
      asm volatile("s_waitcnt lgkmcnt(0)"                                                                        \
                   : "+v"(ka[(F)]), "+v"(ka[(F) + 1]), "+v"(ka[(F) + 2]), "+v"(ka[(F) + 3]), "+v"(va[(F)]),       \
                     "+v"(va[(F) + 1]), "+v"(va[(F) + 2]), "+v"(va[(F) + 3]));                                   \
    } else {                                                                                                     \
      asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(ka[(F)]), "+v"(ka[(F) + 1]), "+v"(va[(F)]), "+v"(va[(F) + 1])); \
    }                                                                                                            \
  } while (0)
#define SEGATTN_DQ_TR_WAIT()                                                                                     \
  do {                                                                                                           \
    if constexpr (NB == 4) {                                                                                     \
      asm volatile("s_waitcnt lgkmcnt(0)"                                                                        \
                   : "+v"(kt[0][0][0]), "+v"(kt[0][0][1]), "+v"(kt[0][1][0]), "+v"(kt[0][1][1]), "+v"(kt[0][2][0]),  \
                     "+v"(kt[0][2][1]), "+v"(kt[0][3][0]), "+v"(kt[0][3][1]), "+v"(kt[1][0][0]), "+v"(kt[1][0][1]),  \
                     "+v"(kt[1][1][0]), "+v"(kt[1][1][1]), "+v"(kt[1][2][0]), "+v"(kt[1][2][1]), "+v"(kt[1][3][0]),  \
                     "+v"(kt[1][3][1]));                                                                         \
    } else {                                                                                                     \
      asm volatile("s_waitcnt lgkmcnt(0)"                                                                        \
                   : "+v"(kt[0][0][0]), "+v"(kt[0][0][1]), "+v"(kt[0][1][0]), "+v"(kt[0][1][1]), "+v"(kt[1][0][0]),  \
                     "+v"(kt[1][0][1]), "+v"(kt[1][1][0]), "+v"(kt[1][1][1]));                                   \
    }                                                                                                            \
  } while (0)

  // Prologue: tiles of steps 0 and 1 on their way, tile 0 landed for everyone.
  fetch_next(0);
  fetch_next(1);
  SEGATTN_VMCNT(kLoadsPerStep);
  __builtin_amdgcn_s_barrier();
  for (int j = 0;;) {
    SEGATTN_DQ_STEP(0);
    if (++j == nsteps) break;
    SEGATTN_DQ_STEP(1);
    if (++j == nsteps) break;
    SEGATTN_DQ_STEP(2);
    if (++j == nsteps) break;
  }
  SEGATTN_VMCNT(0);  // the surplus fetches have landed: the ring may be reused by the next item
#undef SEGATTN_DQ_STEP
#undef SEGATTN_DQ_ROWS_WAIT
#undef SEGATTN_DQ_TR_WAIT
#undef SEGATTN_VMCNT
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
  __shared__ __attribute__((aligned(1024))) unsigned char smem[DqGeom<D>::kBytes];  // ring of [K tile][V tile]
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
  prepare_resolve_divs(p, pa, hs, grid_q);
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
