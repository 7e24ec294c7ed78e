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

#include <atomic>

#include "segattn_bwd_tiles.h"

namespace segattn {

// ---------------------------------------------------------------------------------------------
// dK, dV
// ---------------------------------------------------------------------------------------------
// LDS of the dK/dV kernel: kBufs step buffers of two [32 x D] tiles, then kBufs x 64 row statistics.
template <int D>
struct DkvGeom {
  static constexpr int kTile = BwdTile<D>::kBytes;
  static constexpr int kBuf = 2 * kTile;
  static constexpr int kBufs = 4;
  static constexpr int kStats = kBufs * kBuf;          // byte offset of the statistics
  static constexpr int kStatBytes = 2 * kBwdStep * 4;  // per step
  static constexpr int kBytes = kStats + kBufs * kStatBytes;
};

template <int D>
__global__ __launch_bounds__(256, 1) void bwd_dkv_kernel(const Problem p, const BwdArgs a, const int blocks_per_seg,
                                                         const int n_seg) {
  using T = BwdTile<D>;
  constexpr int NC = D / 16, NB = D / 32;
  constexpr int BK = 128;  // key rows per workgroup
  // A ring of four step buffers, [Q tile][dO tile] each, and behind them the steps' row statistics
  // [32 x -LSE/scale | 32 x delta].  Tiles travel HBM -> LDS with global_load_lds (no staging
  // registers, no LDS stores), three steps ahead of their use.
  using G = DkvGeom<D>;
  constexpr int kTile = G::kTile, kBuf = G::kBuf, NBUF = G::kBufs, kStats = G::kStats, kStatBytes = G::kStatBytes;
  constexpr int LPW = T::kChunks / 8;       // wave-wide 1 KB loads per tensor, step and wave
  constexpr int kLoadsPerStep = 2 * LPW + 1;  // per wave: Q, dO, row statistics
  static_assert((NBUF - 1) * kBuf + kTile + 16 * T::kRowBytes < 65536, "LDS offsets must fit the 16-bit immediate");
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];

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

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int hi = lane >> 5, col = lane & 31, i16 = lane & 15, g16 = (lane >> 4) & 1;
  const float c = p.scale_log2e;
  // this lane's key row (clamped for loads; stores are guarded)
  const long long jw0 = j0 + 32 * wave;
  long long jk = jw0 + col;
  const bool key_ok = jk < j_end;
  jk = key_ok ? jk : j_end - 1;
  const long long koff = ((sq.row0 + jk) * p.Hkv + kv) * D;
  // K^T and V^T operands of this lane's key: only ever MFMA operands, so they are parked in
  // accumulation registers and the vector registers stay free.  V goes in negated: the dP
  // accumulator then starts at delta and ends as delta - dP (one subtraction per element saved),
  // dS and dK come out negated and the sign returns with the final scale.
  bf16x8 Kr[NC], Vr[NC];
#pragma unroll
  for (int kc = 0; kc < NC; ++kc) {
    Kr[kc] = park(*(const uint4 *)(a.k + koff + 16 * kc + 8 * hi));
    uint4 vv = *(const uint4 *)(a.v + koff + 16 * kc + 8 * hi);
    vv.x ^= 0x80008000u;
    vv.y ^= 0x80008000u;
    vv.z ^= 0x80008000u;
    vv.w ^= 0x80008000u;
    Vr[kc] = park(vv);
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

  // ---- HBM -> LDS.  Load i of a wave covers bytes [(wave LPW + i) 1024, +1024) of a tile: row
  // (wave LPW + i) rows-per-KB + lane / chunks, chunk slot lane % chunks, which receives the
  // global chunk slot ^ swz(row) -- the tile's swizzle applied on the global side, since the LDS
  // side of such a load is linear in the lane.  Tiles are fetched in step order (query head
  // major); fetches beyond the last step repeat it (never read), so every wait is one constant.
  const long long head0_q = (sq.row0 * p.Hq + (long long)kv * p.g) * D;   // element offset of (b, row 0, first head)
  const long long head0_s = sq.stat0 + (long long)kv * p.g * sq.stat_stride;
  const unsigned char *const fq0 = (const unsigned char *)(a.q + head0_q + q_begin * q_stride);
  const unsigned char *const fg0 = (const unsigned char *)(a.dout + head0_q + q_begin * q_stride);
  const unsigned row_bytes = (unsigned)(q_stride * 2);
  constexpr int kRowsPerKB = 1024 / T::kRowBytes;
  const int last_rel = (int)(next_end - 1 - q_begin);
  // byte offset of the lane's chunk from the first row of a 32-row tile of one head; for the last
  // step of a head, which can reach past the last query row, with the lane's row clamped
  unsigned f_off[LPW], f_off_last[LPW];
#pragma unroll
  for (int i = 0; i < LPW; ++i) {
    const int row = (wave * LPW + i) * kRowsPerKB + lane / T::kChunks;
    const unsigned chunk = (unsigned)(((lane % T::kChunks) ^ T::swz(row)) << 4);
    const int r_last = (steps_per_head - 1) * kBwdStep + row <= last_rel ? row : last_rel - (steps_per_head - 1) * kBwdStep;
    f_off[i] = (unsigned)row * row_bytes + chunk;
    f_off_last[i] = (unsigned)r_last * row_bytes + chunk;
  }
  // row statistics of a step: lanes 0..31 fetch -LSE/scale, lanes 32..63 delta (4 bytes each)
  const float *const f_stat0 = (lane < kBwdStep ? a.nls : a.delta) + head0_s + q_begin;
  LDS_AS unsigned char *const lds = (LDS_AS unsigned char *)smem;
  const unsigned lds_base = (unsigned)(size_t)lds;
  // fetch cursor: head, step inside the head, and the byte offset of that tile from fq0 / fg0.
  // A fetch comes in three parts (Q tile, dO tile, statistics + cursor advance) so that a step can
  // issue them behind different products.
  int f_head = 0, f_step = 0;
  unsigned long long f_at = 0;
  const float *f_stat = f_stat0;  // row statistic of the cursor's head (per lane: which of the two arrays)
  auto fetch_tile = [&](const unsigned char *base, int lds_off) __attribute__((always_inline)) {
    const bool last = f_step == steps_per_head - 1;
    LDS_AS unsigned char *dst = lds + lds_off + wave * (LPW * 1024);
#pragma unroll
    for (int i = 0; i < LPW; ++i) {
      // (the lane offset passes through an empty asm so that it is widened to 64 bits here, next to the
      // addition: the load then takes a scalar base plus a 32-bit lane offset)
      unsigned off = last ? f_off_last[i] : f_off[i];
      asm volatile("" : "+v"(off));
      __builtin_amdgcn_global_load_lds((const GLB_AS void *)(base + f_at + off), (LDS_AS void *)(dst + i * 1024), 16, 0, 0);
    }
  };
  auto fetch_stats_and_advance = [&](int buf) __attribute__((always_inline)) {
    int r = f_step * kBwdStep + (lane & 31);
    r = r < last_rel ? r : last_rel;
    __builtin_amdgcn_global_load_lds((const GLB_AS void *)(f_stat + r), (LDS_AS void *)(lds + kStats + buf * kStatBytes), 4, 0, 0);
    if (f_step + 1 < steps_per_head) {
      f_step += 1;
      f_at += (unsigned long long)kBwdStep * row_bytes;
    } else if (f_head + 1 < p.g) {
      f_step = 0;
      f_head += 1;
      f_at = (unsigned long long)f_head * (D * 2);
      f_stat += sq.stat_stride;
    }
  };
  auto fetch_next = [&](int buf) __attribute__((always_inline)) {
    fetch_tile(fq0, buf * kBuf);
    fetch_tile(fg0, buf * kBuf + kTile);
    fetch_stats_and_advance(buf);
  };
#define SEGATTN_VMCNT(N) __builtin_amdgcn_s_waitcnt(0x0F70 | ((N) & 15) | (((N) >> 4) << 14))

  // ---- per-lane LDS read addresses inside a step buffer (the buffer and the tensor are immediates)
  // row operands: tile row `col`, logical chunk 2 kc + hi
  unsigned ro[NC];
#pragma unroll
  for (int kc = 0; kc < NC; ++kc) ro[kc] = lds_base + (unsigned)T::at(col, 2 * kc + hi);
  // transposed operands (see read_transposed): rows 4 hi + i16/4 (+ 8 u + 16 h2), chunk 4 nb + 2 g16 +
  // (i16 % 4) / 2; the swizzle is the same for rows 16 apart, so h2 is an immediate
  unsigned tro[NB][2];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb)
#pragma unroll
    for (int u = 0; u < 2; ++u)
      tro[nb][u] = lds_base + (unsigned)(T::at(4 * hi + (i16 >> 2) + 8 * u, 4 * nb + 2 * g16 + ((i16 & 3) >> 1)) + 8 * (i16 & 1));
  static_assert(T::swz(0) == T::swz(16) && T::swz(5) == T::swz(21) && T::swz(15) == T::swz(31), "h2 as an immediate");
  // row statistics of the lane's 16 query rows: rows 8 g4 + 4 hi .. +3
  const unsigned sto = lds_base + (unsigned)(kStats + 16 * hi);

  typedef int i32x4 __attribute__((ext_vector_type(4)));
  typedef float f32x2 __attribute__((ext_vector_type(2)));
  // Q row operands and row statistics (-LSE/scale, delta of the lane's 16 query rows) of the current
  // step, read behind the last products of the step before
  i32x4 qa[NC], st_s[4], st_d[4];
  auto qa_wait = [&]() __attribute__((always_inline)) {
    if constexpr (NC == 8) {
      asm volatile("s_waitcnt lgkmcnt(0)"
                   : "+v"(qa[0]), "+v"(qa[1]), "+v"(qa[2]), "+v"(qa[3]), "+v"(qa[4]), "+v"(qa[5]), "+v"(qa[6]), "+v"(qa[7]),
                     "+v"(st_s[0]), "+v"(st_s[1]), "+v"(st_s[2]), "+v"(st_s[3]), "+v"(st_d[0]), "+v"(st_d[1]), "+v"(st_d[2]),
                     "+v"(st_d[3]));
    } else {
      asm volatile("s_waitcnt lgkmcnt(0)"
                   : "+v"(qa[0]), "+v"(qa[1]), "+v"(qa[2]), "+v"(qa[3]), "+v"(st_s[0]), "+v"(st_s[1]), "+v"(st_s[2]),
                     "+v"(st_s[3]), "+v"(st_d[0]), "+v"(st_d[1]), "+v"(st_d[2]), "+v"(st_d[3]));
    }
  };

  int i_rel0 = 0;  // first query of the step, relative to q_begin
  // One step on the tile in buffer B, laid out by hand as 32 slots of one matrix product each; the
  // LDS reads and the vector-ALU work of the step are spread over the slots so that they issue in
  // the shadow of the products (a product occupies the matrix pipe for 32 cycles; about six vector
  // instructions fit under it).  On entry qa holds the Q row operands of the tile.
  //   slots  0.. 7   S' = Q K^T - LSE/scale (the accumulator starts at -LSE/scale, so that
  //                  P = exp2(S' c) needs no subtraction); reads: dO row operands; the tile three
  //                  steps on is requested (its buffer was last read before the previous barrier)
  //   slots  8..15   dP' = delta - dO V^T (the accumulator starts at delta, V is negated);
  //                  P of the first 16 queries (exp2, bf16) and the exponentials of two more;
  //                  reads: transposed operands of the first 16 queries
  //   slots 16..23   first 16 queries: dV^T += dO^T P (four products, dS' = P dP' formed behind
  //                  them), dK'^T += Q^T dS' (four); P, dS' of the other 16 queries; reads: their
  //                  transposed operands
  //   barrier        the tile of the next step has landed for every wave; nobody reads this
  //                  step's tile any more
  //   slots 24..31   the other 16 queries; reads: Q row operands and row statistics of the next step
  // A tile that holds pairs outside [q_lo, q_lim) (the diagonal of the keys' own segment, the end of
  // the query range) gets their scores set to -inf before the exponentials: weight exactly 0.
#define SEGATTN_DKV_EXP(r) pe[r] = __builtin_amdgcn_exp2f(S[r] * c)
#define SEGATTN_DKV_PPAIR(r) /* P of rows r, r+1 as a bf16 pair */                                               \
  Pw[(r) / 2] = __builtin_bit_cast(int, __builtin_convertvector((f32x2){pe[r], pe[(r) + 1]}, bf16x2))
#define SEGATTN_DKV_DSPAIR(r) /* dS' of rows r, r+1 as a bf16 pair */                                            \
  dSw[(r) / 2] = __builtin_bit_cast(int, __builtin_convertvector((f32x2){pe[r] * dP[r], pe[(r) + 1] * dP[(r) + 1]}, bf16x2))
#define SEGATTN_DKV_STEP(B)                                                                                      \
  do {                                                                                                           \
    constexpr int BO = (B) * kBuf, BN = (((B) + 1) % NBUF) * kBuf, BF = ((B) + NBUF - 1) % NBUF;                 \
    constexpr int SN = (((B) + 1) % NBUF) * kStatBytes; /* statistics of the next step */                        \
    const bool plain = i_rel0 >= q_lo_max && i_rel0 + kBwdStep <= q_lim_min; /* every pair of the tile counts */ \
    i32x4 ga[NC];                                                                                                \
    s16x4 gt[NB][2], qt[NB][2], gu[NB][2], qu[NB][2];                                                            \
    float pe[16];                                                                                                \
    int Pw[8], dSw[8];                                                                                           \
    f32x16 S, dP; /* the accumulators start at -LSE/scale and at delta of the rows */                            \
    _Pragma("unroll") for (int r = 0; r < 16; ++r) {                                                             \
      S[r] = __int_as_float(st_s[r / 4][r % 4]);                                                                 \
      dP[r] = __int_as_float(st_d[r / 4][r % 4]);                                                                \
    }                                                                                                            \
    __builtin_amdgcn_sched_barrier(0);                                                                           \
    _Pragma("unroll") for (int kc = 0; kc < NC; ++kc) { /* slots 0 .. NC-1 */                                    \
      S = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, qa[kc]), Kr[kc], S, 0, 0, 0);       \
      __builtin_amdgcn_sched_barrier(0);                                                                         \
      /* reads early in the chain, so that the wait behind it is free; then the request for the tile two        \
         steps on, in three parts */                                                                             \
      if (kc < NC / 2) {                                                                                         \
        asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(ga[2 * kc]) : "v"(ro[2 * kc]), "n"(BO + kTile));     \
        asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(ga[2 * kc + 1]) : "v"(ro[2 * kc + 1]), "n"(BO + kTile)); \
      }                                                                                                          \
      if (kc == NC / 2) fetch_tile(fq0, BF * kBuf);                                                              \
      if (kc == NC / 2 + 1) fetch_tile(fg0, BF * kBuf + kTile);                                                  \
      if (kc == NC - 1) fetch_stats_and_advance(BF);                                                             \
      __builtin_amdgcn_sched_barrier(0);                                                                         \
    }                                                                                                            \
    SEGATTN_DKV_WAIT_A();                                                                                        \
    __builtin_amdgcn_sched_barrier(0);                                                                           \
    _Pragma("unroll") for (int kc = 0; kc < NC; ++kc) { /* slots NC .. 2 NC-1 */                                 \
      dP = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, ga[kc]), Vr[kc], dP, 0, 0, 0);     \
      __builtin_amdgcn_sched_barrier(0);                                                                         \
      /* reads: transposed operands of the first 16 queries, dO^T (used first) before Q^T */                     \
      if (kc < NB) {                                                                                             \
        _Pragma("unroll") for (int u = 0; u < 2; ++u)                                                            \
          asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(gt[kc][u]) : "v"(tro[kc][u]), "n"(BO + kTile)); \
        _Pragma("unroll") for (int u = 0; u < 2; ++u)                                                            \
          asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(qt[kc][u]) : "v"(tro[kc][u]), "n"(BO));      \
      }                                                                                                          \
      if (kc == 0 && __builtin_expect(!plain, 0)) { /* rare: laid out off the step's straight path */            \
        _Pragma("unroll") for (int r = 0; r < 16; ++r) {                                                         \
          const int i_rel = i_rel0 + 8 * (r / 4) + 4 * hi + r % 4; /* query row, relative to q_begin */          \
          S[r] = ((i_rel >= q_lo) & (i_rel < q_lim)) ? S[r] : -INFINITY;                                         \
        }                                                                                                        \
      }                                                                                                          \
      /* exponentials: NC = 8: rows 0..7 one per slot, rows 8, 9 in the last two; NC = 4: two per slot */        \
      if (NC == 8) {                                                                                             \
        SEGATTN_DKV_EXP(kc);                                                                                     \
        if (kc >= 6) SEGATTN_DKV_EXP(kc + 2);                                                                    \
        if (kc & 1) SEGATTN_DKV_PPAIR(kc - 1);                                                                   \
      } else {                                                                                                   \
        SEGATTN_DKV_EXP(2 * kc);                                                                                 \
        SEGATTN_DKV_EXP(2 * kc + 1);                                                                             \
        SEGATTN_DKV_PPAIR(2 * kc);                                                                               \
        if (kc >= 2) { SEGATTN_DKV_EXP(2 * kc + 4); SEGATTN_DKV_EXP(2 * kc + 5); }                               \
      }                                                                                                          \
      __builtin_amdgcn_sched_barrier(0);                                                                         \
    }                                                                                                            \
    SEGATTN_TR_WAIT(gt, qt);                                                                                     \
    const bf16x8 P0 = __builtin_bit_cast(bf16x8, (i32x4){Pw[0], Pw[1], Pw[2], Pw[3]});                           \
    bf16x8 dS0;                                                                                                  \
    /* slots 2 NC .. 2 NC + 2 NB - 1: first 16 queries */                                                        \
    _Pragma("unroll") for (int t = 0; t < 2 * NB; ++t) {                                                         \
      if (t < NB) {                                                                                              \
        mma_acc(dVa[t], tr_pair(gt[t]), P0);                                                                     \
      } else {                                                                                                   \
        if (t == NB) dS0 = __builtin_bit_cast(bf16x8, (i32x4){dSw[0], dSw[1], dSw[2], dSw[3]});                  \
        mma_acc(dKa[t - NB], tr_pair(qt[t - NB]), dS0);                                                          \
      }                                                                                                          \
      __builtin_amdgcn_sched_barrier(0);                                                                         \
      /* reads: transposed operands of the other 16 queries, dO^T first (their registers: after the dV          \
         products nothing reads gt any more) */                                                                  \
      if (t >= NB / 2 && t < NB / 2 + NB) {                                                                      \
        const int nb = t - NB / 2;                                                                               \
        _Pragma("unroll") for (int u = 0; u < 2; ++u) {                                                          \
          asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(gu[nb][u]) : "v"(tro[nb][u]), "n"(BO + kTile + 16 * T::kRowBytes)); \
          asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(qu[nb][u]) : "v"(tro[nb][u]), "n"(BO + 16 * T::kRowBytes)); \
        }                                                                                                        \
      }                                                                                                          \
      /* vector ALU: dS' of the first 16 queries behind the first dV products, then the other 16 queries */      \
      if (NB == 4) {                                                                                             \
        if (t == 0) { SEGATTN_DKV_DSPAIR(0); SEGATTN_DKV_DSPAIR(2); }                                            \
        if (t == 1) { SEGATTN_DKV_DSPAIR(4); SEGATTN_DKV_DSPAIR(6); }                                            \
        if (t >= 2) SEGATTN_DKV_EXP(8 + t); /* rows 10 .. 15 */                                                  \
        if (t == 3) { SEGATTN_DKV_PPAIR(8); SEGATTN_DKV_DSPAIR(8); }                                             \
        if (t == 4) { SEGATTN_DKV_PPAIR(10); SEGATTN_DKV_DSPAIR(10); }                                           \
        if (t == 6) { SEGATTN_DKV_PPAIR(12); SEGATTN_DKV_DSPAIR(12); }                                           \
      } else {                                                                                                   \
        if (t == 0) { SEGATTN_DKV_DSPAIR(0); SEGATTN_DKV_DSPAIR(2); SEGATTN_DKV_DSPAIR(4); SEGATTN_DKV_DSPAIR(6); } \
        if (t == 1) { SEGATTN_DKV_EXP(12); SEGATTN_DKV_EXP(13); SEGATTN_DKV_PPAIR(8); SEGATTN_DKV_DSPAIR(8); }   \
        if (t == 2) { SEGATTN_DKV_EXP(14); SEGATTN_DKV_EXP(15); SEGATTN_DKV_PPAIR(10); SEGATTN_DKV_DSPAIR(10); } \
        if (t == 3) { SEGATTN_DKV_PPAIR(12); SEGATTN_DKV_DSPAIR(12); }                                           \
      }                                                                                                          \
      __builtin_amdgcn_sched_barrier(0);                                                                         \
    }                                                                                                            \
    SEGATTN_DKV_PPAIR(14);                                                                                       \
    SEGATTN_DKV_DSPAIR(14);                                                                                      \
    const bf16x8 P1 = __builtin_bit_cast(bf16x8, (i32x4){Pw[4], Pw[5], Pw[6], Pw[7]});                           \
    const bf16x8 dS1 = __builtin_bit_cast(bf16x8, (i32x4){dSw[4], dSw[5], dSw[6], dSw[7]});                      \
    i_rel0 += kBwdStep;                                                                                          \
    if (i_rel0 >= steps_per_head * kBwdStep) i_rel0 = 0;                                                         \
    SEGATTN_TR_WAIT(gu, qu);                                                                                     \
    __builtin_amdgcn_sched_barrier(0);                                                                           \
    SEGATTN_VMCNT(2 * kLoadsPerStep); /* the next step's tile has landed (this wave's part) */                   \
    __builtin_amdgcn_s_barrier(); /* ... and everyone's; nobody reads this step's tile any more */               \
    __builtin_amdgcn_sched_barrier(0);                                                                           \
    /* slots .. 31: the other 16 queries; behind them the Q row operands of the next step */                     \
    _Pragma("unroll") for (int t = 0; t < 2 * NB; ++t) {                                                         \
      if (t < NB) mma_acc(dVa[t], tr_pair(gu[t]), P1);                                                           \
      else mma_acc(dKa[t - NB], tr_pair(qu[t - NB]), dS1);                                                       \
      __builtin_amdgcn_sched_barrier(0);                                                                         \
      if (t < NB) { /* in the first half of the slots: 2 NC / NB row operands, two of each statistic */          \
        _Pragma("unroll") for (int e = 0; e < NC / NB; ++e)                                                      \
          asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(qa[t * (NC / NB) + e]) : "v"(ro[t * (NC / NB) + e]), "n"(BN)); \
        _Pragma("unroll") for (int e = 0; e < 4 / NB; ++e) {                                                     \
          const int g4 = t * (4 / NB) + e;                                                                       \
          asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(st_s[g4]) : "v"(sto), "n"(SN + 32 * g4));          \
          asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(st_d[g4]) : "v"(sto), "n"(SN + 128 + 32 * g4));    \
        }                                                                                                        \
      }                                                                                                          \
      __builtin_amdgcn_sched_barrier(0);                                                                         \
    }                                                                                                            \
    qa_wait();                                                                                                   \
  } while (0)
  // everything read in slots 0 .. NC-1 has arrived
#define SEGATTN_DKV_WAIT_A()                                                                                     \
  do {                                                                                                           \
    if constexpr (NC == 8) {                                                                                     \
      asm volatile("s_waitcnt lgkmcnt(0)"                                                                        \
                   : "+v"(ga[0]), "+v"(ga[1]), "+v"(ga[2]), "+v"(ga[3]), "+v"(ga[4]), "+v"(ga[5]), "+v"(ga[6]), "+v"(ga[7])); \
    } else {                                                                                                     \
      asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(ga[0]), "+v"(ga[1]), "+v"(ga[2]), "+v"(ga[3]));                 \
    }                                                                                                            \
  } while (0)
#define SEGATTN_TR_WAIT(G, Q)                                                                                    \
  do {                                                                                                           \
    if constexpr (NB == 4) {                                                                                     \
      asm volatile("s_waitcnt lgkmcnt(0)"                                                                        \
                   : "+v"(G[0][0]), "+v"(G[0][1]), "+v"(G[1][0]), "+v"(G[1][1]), "+v"(G[2][0]), "+v"(G[2][1]),   \
                     "+v"(G[3][0]), "+v"(G[3][1]), "+v"(Q[0][0]), "+v"(Q[0][1]), "+v"(Q[1][0]), "+v"(Q[1][1]),   \
                     "+v"(Q[2][0]), "+v"(Q[2][1]), "+v"(Q[3][0]), "+v"(Q[3][1]));                                \
    } else {                                                                                                     \
      asm volatile("s_waitcnt lgkmcnt(0)"                                                                        \
                   : "+v"(G[0][0]), "+v"(G[0][1]), "+v"(G[1][0]), "+v"(G[1][1]), "+v"(Q[0][0]), "+v"(Q[0][1]),   \
                     "+v"(Q[1][0]), "+v"(Q[1][1]));                                                              \
    }                                                                                                            \
  } while (0)
  auto tr_pair = [](const s16x4(&h)[2]) __attribute__((always_inline)) {
    return __builtin_bit_cast(bf16x8, __builtin_shufflevector(h[0], h[1], 0, 1, 2, 3, 4, 5, 6, 7));
  };
  // Prologue: tiles of steps 0, 1 and 2 on their way, tile 0 landed for everyone, its Q row operands read.
  fetch_next(0);
  fetch_next(1);
  fetch_next(2);
  SEGATTN_VMCNT(2 * kLoadsPerStep);
  __builtin_amdgcn_s_barrier();
#pragma unroll
  for (int kc = 0; kc < NC; ++kc) asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(qa[kc]) : "v"(ro[kc]), "n"(0));
#pragma unroll
  for (int g4 = 0; g4 < 4; ++g4) {
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(st_s[g4]) : "v"(sto), "n"(32 * g4));
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(st_d[g4]) : "v"(sto), "n"(128 + 32 * g4));
  }
  qa_wait();
  for (int it = 0;;) {
    SEGATTN_DKV_STEP(0);
    if (++it == nsteps) break;
    SEGATTN_DKV_STEP(1);
    if (++it == nsteps) break;
    SEGATTN_DKV_STEP(2);
    if (++it == nsteps) break;
    SEGATTN_DKV_STEP(3);
    if (++it == nsteps) break;
  }
  SEGATTN_VMCNT(0);  // the surplus fetches have landed before the workgroup gives up its LDS
#undef SEGATTN_DKV_STEP
#undef SEGATTN_DKV_EXP
#undef SEGATTN_DKV_PPAIR
#undef SEGATTN_DKV_DSPAIR
#undef SEGATTN_DKV_WAIT_A
#undef SEGATTN_TR_WAIT
#undef SEGATTN_VMCNT
  if (!key_ok) return;
  const float back = -p.scale;  // dK' = -dK (see the negated V operands)
#pragma unroll
  for (int nb = 0; nb < NB; ++nb)
#pragma unroll
    for (int rg = 0; rg < 4; ++rg) {
      const int d = 32 * nb + 8 * rg + 4 * hi;
      const f32x4 gk = {dKa[nb][4 * rg + 0] * back, dKa[nb][4 * rg + 1] * back,
                        dKa[nb][4 * rg + 2] * back, dKa[nb][4 * rg + 3] * back};
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
  // the ring of step buffers exceeds the 64 KB a kernel gets without asking (head_dim 128)
  static std::atomic<bool> ready{false};
  if (!ready.load(std::memory_order_acquire)) {
    const hipError_t e = hipFuncSetAttribute((const void *)bwd_dkv_kernel<D>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                             DkvGeom<D>::kBytes);
    if (e != hipSuccess) return e;
    ready.store(true, std::memory_order_release);
  }
  hipLaunchKernelGGL(bwd_dkv_kernel<D>, dim3((unsigned)grid_k), dim3(256), DkvGeom<D>::kBytes, st, p, a, blocks_per_seg,
                     n_seg);
  return hipGetLastError();
}

hipError_t launch_bwd_mfma(const Problem &p, const BwdArgs &a, hipStream_t st) {
  const hipError_t e = launch_bwd_dq(p, a, st);
  if (e != hipSuccess) return e;
  return p.D == 128 ? launch_dkv<128>(p, a, st) : launch_dkv<64>(p, a, st);
}

}  // namespace segattn
