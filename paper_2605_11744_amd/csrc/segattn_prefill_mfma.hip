// bf16 MFMA prefill kernel of libsegattn: segment-level causal attention (Eq. 12 with the
// per-head context of Eq. 13, Appendix C) for gfx950.
//
// Workgroup = 8 waves (two per SIMD, 256 registers each) for head_dim 128, 4 waves for head_dim
// 64 (152 registers: three workgroups share a CU).  HS query heads of one GQA group share the
// staged K/V rows; each wave owns one head and 32 consecutive query rows.  Keys are consumed in
// steps of 32:
//
//   S^T[key][query] = K_step . Q^T      v_mfma_f32_32x32x16_bf16, A = K rows read from LDS
//   P = exp2(S^T c - m c)               per query, m a running reference maximum
//   O^T[d][query] += V_step^T . P^T     A = V^T via ds_read_b64_tr_b16, B = P taken straight
//                                       from the S^T accumulator registers
//
// Computing the transposed products makes the accumulator layout of S^T (lane = query, the
// lane's registers = keys) exactly the B-operand layout of the second product, so P never
// leaves the register file.
//
// The loop is software-pipelined over three consecutive steps: while the matrix cores
// compute S^T of step j+1 and the PV product of step j-1, the vector ALU turns S^T of step j
// into P (one exp2, one fma, half a max3, half a convert and half a dot2 per element: about
// 21 issue cycles per 32-cycle MFMA).  The reference maximum is lazy: P of a step is formed
// with the maximum known so far; only if the step's own maximum exceeds it by more than 2^8
// (checked before that P is used) are the accumulators rescaled and that P recomputed, so
// the common path has no accumulator rescale and exp2 never overflows.
//
// K/V rows travel HBM -> LDS with global_load_lds_dwordx4 (no staging registers) into a ring
// of step slots, three or more steps ahead of their use (eight-wave workgroups: 8 slots, the
// waves meet at a barrier only every other step and fetch two steps there; otherwise 5 slots and
// a barrier per step); the 16-byte chunks of a row are XOR-swizzled by the loading lanes so that
// both the row-wise K reads and the transposing V reads
// are free of bank conflicts.  Steps that need an element mask (the diagonal of the query's
// own segment, the ragged end of a span) run the same pipelined step with the mask applied to
// S^T first, and the loader keeps a constant number of loads in flight to the very end (it
// fetches the last step again once it runs out), so one kind of step with one fixed wait covers
// the whole key range; a wave that has passed its last query only keeps loading and meeting at
// the barriers until the other waves of the workgroup are done.  Paths outside that step matter
// more than their share of the arithmetic suggests: a register spilled there is reloaded
// through the same counter the K/V prefetch uses, and waiting for it drains the prefetch queue.
#include <atomic>
#include <mutex>

#include <type_traits>

#include "segattn_work.h"

namespace segattn {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
#define LDS_AS __attribute__((address_space(3)))
#define GLB_AS __attribute__((address_space(1)))

constexpr int kStepKeys = 32;
// LDS ring of step slots.  Per-step sync: steps j-1 .. j+3 are resident or in flight (5 slots, one
// step of loads may still be in flight at a sync).  Pair sync (eight-wave workgroups): the waves
// meet only at every other step and fetch two steps there; steps j-1 .. j+6 (8 slots, two steps in
// flight at a sync).
__host__ __device__ constexpr bool pair_sync(int nw, int qb) {
#ifdef SEGATTN_PREFILL_STEP_SYNC
  return false;
#else
  return nw == 8 && qb == 1;
#endif
}
__host__ __device__ constexpr int ring_slots(int nw, int qb) { return pair_sync(nw, qb) ? 8 : 5; }
constexpr float kLazyLimit = 256.f;  // a lane's 16-weight row sum above this triggers a rescale

template <int D>
struct StepGeom {
  static constexpr int kRowBytes = 2 * D;
  static constexpr int kChunks = D / 8;                        // 16-byte chunks per row
  static constexpr int kTensorBytes = kStepKeys * kRowBytes;   // K (or V) rows of one step
  static constexpr int kSlotBytes = 2 * kTensorBytes;
  static constexpr int kInstr = kTensorBytes / 1024;           // wave-wide 1 KB loads per tensor
  static constexpr int kRowsPerInstr = 1024 / kRowBytes;
  static constexpr int kRowsPer256 = 256 / kRowBytes;          // rows sharing one 64-bank window
  // K rows are read 16 lanes = 16 consecutive rows at one logical chunk: XOR-ing all chunk bits
  // with the row (four bits for 256-byte rows) spreads the 16 rows over all 64 banks.  (With the
  // low three bits only, rows r and r + 8 met in one bank: a two-way conflict on every K read.)
  __device__ static constexpr int swz_k(int row) { return (row / kRowsPer256) & (kChunks - 1) & 15; }
  __device__ static constexpr int swz_v(int row) { return 4 * ((row / kRowsPer256) % (kChunks / 4)); }
};

__device__ inline float half_max(float x) {  // max over lanes l and l^32
  const int xi = __float_as_int(x);
  const auto sw = __builtin_amdgcn_permlane32_swap(xi, xi, false, false);
  return fmaxf(__int_as_float(sw[0]), __int_as_float(sw[1]));
}
__device__ inline float half_sum(float x) {
  const int xi = __float_as_int(x);
  const auto sw = __builtin_amdgcn_permlane32_swap(xi, xi, false, false);
  return __int_as_float(sw[0]) + __int_as_float(sw[1]);
}

// QB = 32-query blocks per wave (1 in every instantiation in use; a head_dim-64 form with 2, one
// wave per SIMD, was 6 to 40 % slower than three 32-row workgroups per CU), NW = waves per
// workgroup.  (D, QB, NW) = (128, 1, 8): two
// waves per SIMD share the issue slots -- while one is blocked behind a matrix product or a
// wait the other issues its softmax -- at the price of reading every K/V operand from LDS for
// half as many products.  All products are compiler builtins in VGPR form (the file is built
// with -amdgpu-mfma-vgpr-form): the compiler sees every MFMA hazard.  An earlier version kept
// O^T in accumulation registers through inline-asm products; wherever the register allocator
// then moved O^T at a control-flow merge, the move could read an accumulator whose product
// was still in the pipeline, and results depended on register allocation.
template <int D, int HS, int QB, int NW>
__device__ __forceinline__ unsigned prefill_mfma_item(const Problem &p, const PrefillArgs &a, const int bid,
                                                      unsigned char *const smem, unsigned *const next_from) {
  // next_from: nullptr, or the queue counter this workgroup takes its next item from.  Thread 0
  // draws the ticket while the output is still being written and hands it back (other threads: 0),
  // so the round trip is over by the time the next round starts.
  using G = StepGeom<D>;  // NW = waves per workgroup; NW * QB = 4 leaves room for two workgroups per CU
  constexpr int RW = 32 * QB;       // query rows per wave
  constexpr int BQ = (NW / HS) * RW; // query rows per workgroup
  constexpr int NC = D / 16;        // k-chunks of the QK^T product
  constexpr int NB = D / 32;        // 32-row blocks of O^T
  constexpr int LPW = G::kInstr / NW;  // wave-wide 1 KB loads per tensor, step and wave
  constexpr bool kPair = pair_sync(NW, QB);
  constexpr int kSlots = ring_slots(NW, QB);
  constexpr int kAhead = kPair ? 2 : 1;  // whole steps of loads that may still be in flight at a sync
  static_assert(LPW >= 1, "too many waves for this tile");

  WorkItem w = resolve(p, a, bid, BQ, HS);
  if (!w.valid) return (next_from && threadIdx.x == 0) ? atomicAdd(next_from, 1u) : 0u;
  pin_uniform(w);

  int tid = threadIdx.x;
  asm volatile("" : "+v"(tid));  // not a loop invariant of the caller's loop (see prefill_mfma_kernel)
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
  const int hi = lane >> 5, col = lane & 31;
  const int i16 = lane & 15, g16 = (lane >> 4) & 1;
  const int head = w.kv * p.g + w.hsub * HS + (wave % HS);
  const int tw0 = w.t0 + (wave / HS) * RW;  // first query row of this wave
  const int ohead = w.ohead0 + (wave % HS);  // the same head where this workgroup's output goes
  const int last_row = w.nq - 1;
  const float c = p.scale_log2e;

  // ---- step schedule (workgroup) and this wave's share of it
  const int n1_needed = (w.t0 + BQ < w.n1) ? (w.t0 + BQ) : w.n1;
  const int nst0 = (w.n0 + kStepKeys - 1) / kStepKeys;
  const int nst1 = (n1_needed + kStepKeys - 1) / kStepKeys;
  const int n = nst0 + nst1;
  int f;  // leading steps that need no element mask for this wave
  if (w.n0 % kStepKeys) {
    f = nst0 - 1;
  } else {
    const int full1 = (tw0 + 1) / kStepKeys;  // span-1 steps whose keys all precede every query
    f = nst0 + (full1 < nst1 ? full1 : nst1);
  }
  int n_act;  // steps at or beyond this one start after the wave's last query: nothing to compute
  {
    const int s1 = (tw0 + RW - 1) / kStepKeys + 1;
    n_act = nst0 + (s1 < nst1 ? s1 : nst1);
  }

  // ---- HBM -> LDS.  Load i of a wave covers LDS bytes [(wave*LPW+i)*1024, +1024) of a tensor:
  //      row r = (wave*LPW+i)*rowsPerInstr + lane/chunks, chunk slot lane%chunks, which receives
  //      global chunk (slot ^ swizzle(r)).  For a full step the lane's byte offset from the
  //      step's first row is a per-span constant (off_k / off_v).
  unsigned off_k[LPW], off_v[LPW];
  LDS_AS unsigned char *const lds = (LDS_AS unsigned char *)smem;
  constexpr int kRing = kSlots * G::kSlotBytes;
  auto next_slot = [](int off) __attribute__((always_inline)) { return off + G::kSlotBytes == kRing ? 0 : off + G::kSlotBytes; };

  // loader state: the step the next loads fetch, where its rows start, how many rows its span
  // has left.  The loader never stops: once the last step has been fetched it keeps fetching
  // that step again (into slots nobody reads any more), so the number of loads in flight at a
  // sync is the same constant at every step and the waits need no case analysis.
  int ld_js = 0, ld_span = -1, ld_left = 0, ld_slot = 0;
  int ld_full_end = 0;  // first step at or after ld_js that is not a plain full step of the loader's span
  const unsigned char *ld_kp = nullptr, *ld_vp = nullptr;
  unsigned ld_stride = 0;
  // Lane offsets of the step's loads (recomputed from the lane index where needed rather than
  // kept in registers through the loop); rows past a ragged end are clamped.
  auto set_offsets = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < LPW; ++i) {
      const int row = (wave * LPW + i) * G::kRowsPerInstr + lane / G::kChunks;
      const int slot_chunk = lane % G::kChunks;
      const int r = (ld_left >= kStepKeys || row < ld_left) ? row : ld_left - 1;
      off_k[i] = (unsigned)r * ld_stride + (unsigned)((slot_chunk ^ G::swz_k(row)) * 16);
      off_v[i] = (unsigned)r * ld_stride + (unsigned)((slot_chunk ^ G::swz_v(row)) * 16);
    }
  };
  // (No lambda below is reached through two different closures: merged call sites would turn
  // the captured state into memory accessed through a pointer chosen at run time.)
  auto span_scalars = [&](int s1) __attribute__((always_inline)) {
    ld_span = s1;
    ld_kp = (const unsigned char *)(s1 ? w.k1 : w.k0);
    ld_vp = (const unsigned char *)(s1 ? w.v1 : w.v0);
    ld_left = s1 ? w.n1 : w.n0;
    ld_stride = (unsigned)((s1 ? w.stride1 : w.stride0) * 2);
    ld_full_end = (s1 ? nst0 : 0) + ld_left / kStepKeys;
    if (ld_full_end > n) ld_full_end = n;
  };
  span_scalars(nst0 > 0 ? 0 : 1);
  set_offsets();
  auto issue_loads = [&]() __attribute__((always_inline)) {  // enqueue the loads of the loader's step into the next ring slot
    LDS_AS unsigned char *dst = lds + ld_slot + wave * (LPW * 1024);
#pragma unroll
    for (int i = 0; i < LPW; ++i) {
      // (the lane offsets pass through an empty asm so that their widening to 64 bits happens here,
      // next to the addition: the load then takes a scalar base plus a 32-bit lane offset, and no
      // vector instruction is spent on its address)
      asm volatile("" : "+v"(off_k[i]), "+v"(off_v[i]));
      __builtin_amdgcn_global_load_lds((const GLB_AS void *)(ld_kp + off_k[i]), (LDS_AS void *)(dst + i * 1024), 16, 0, 0);
      __builtin_amdgcn_global_load_lds((const GLB_AS void *)(ld_vp + off_v[i]),
                                       (LDS_AS void *)(dst + G::kTensorBytes + i * 1024), 16, 0, 0);
    }
    ld_slot = next_slot(ld_slot);
  };
  // Branch-free advance for the hot loop: the caller guarantees that the next step is a plain
  // full step of the same span (ld_js + 1 < ld_full_end).
  auto loader_advance_plain = [&]() __attribute__((always_inline)) {
    ld_js += 1;
    ld_kp += (size_t)kStepKeys * ld_stride;
    ld_vp += (size_t)kStepKeys * ld_stride;
    ld_left -= kStepKeys;
  };
  auto loader_advance = [&]() __attribute__((always_inline)) {  // move on to the next step, if there is one (uniform branches)
    ld_js += 1;
    if (ld_js < n) {
      const bool to_span1 = ld_span == 0 && ld_js == nst0;
      if (to_span1) {
        ld_span = 1;
        ld_kp = (const unsigned char *)w.k1;
        ld_vp = (const unsigned char *)w.v1;
        ld_left = w.n1;
        ld_stride = (unsigned)(w.stride1 * 2);
        ld_full_end = nst0 + ld_left / kStepKeys;
        if (ld_full_end > n) ld_full_end = n;
      } else {
        ld_kp += (size_t)kStepKeys * ld_stride;
        ld_vp += (size_t)kStepKeys * ld_stride;
        ld_left -= kStepKeys;
      }
      if (to_span1 || ld_left < kStepKeys) set_offsets();
    }
  };
  // s_waitcnt vmcnt: at most kAhead whole steps of this wave's loads stay in flight
  static_assert(kAhead * 2 * LPW < 64, "vmcnt is a 6-bit counter");
#define SEGATTN_VMCNT(N) __builtin_amdgcn_s_waitcnt(0x0F70 | ((N) & 15) | (((N) >> 4) << 14))
  // The sync of step j, executed by every wave in the middle of the step (in the prologue for
  // j = 0).  Per-step form: the loads of steps <= j+2 have landed for every wave and every wave is
  // done reading the slot of step j-1, which now receives the loads of step j+4.  Pair form: only
  // even steps sync; the loads of steps <= j+3 have landed (the odd step that follows needs j+2
  // and j+3 and meets nobody) and the slots of steps j-2 and j-1 receive steps j+6 and j+7.
  // The loader is left at the last step fetched; the caller moves it on once more.
  auto sync_step = [&]() __attribute__((always_inline)) {
    SEGATTN_VMCNT(kAhead * 2 * LPW);
    __builtin_amdgcn_s_barrier();
    issue_loads();
    if constexpr (kPair) {
      loader_advance();
      issue_loads();
    }
  };

  for (int i = 0; i < (kPair ? kSlots - 2 : kSlots - 1); ++i) {
    issue_loads();
    loader_advance();
  }

  // ---- Q^T operands: Qr[qb][kc] = Q[row(qb, col)][16 kc + 8 hi .. +7]
  bf16x8 Qr[QB][NC];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    int t = tw0 + 32 * qb + col;
    t = t < last_row ? t : last_row;
    const unsigned short *qrow = w.q + ((long long)t * p.Hq + head) * D + 8 * hi;
#pragma unroll
    for (int kc = 0; kc < NC; ++kc) {
      const i32x4 v = __builtin_bit_cast(i32x4, *(const uint4 *)(qrow + 16 * kc));
      Qr[qb][kc] = __builtin_bit_cast(bf16x8, v);
    }
  }

  // ---- per-lane LDS read offsets inside a slot
  // K operand of k-chunk kc: row col, logical chunk 2 kc + hi, swizzled with the row: one lane
  // address per k-chunk
  constexpr int NKA = NC;
  static_assert(NC <= 8, "one lane address per k-chunk");
  int koff[NKA];
#pragma unroll
  for (int i = 0; i < NKA; ++i) koff[i] = col * G::kRowBytes + (((2 * i + hi) ^ G::swz_k(col)) << 4);
  int voff[NB];  // V^T operand: row 4hi + i16/4 (+16 h2 + 8 u), columns 32 nb + 16 g16 + 4 (i16%4) ..+3
  {
    const int vrow = 4 * hi + (i16 >> 2);
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      const int chunk = 4 * nb + 2 * g16 + ((i16 & 3) >> 1);
      voff[nb] = G::kTensorBytes + vrow * G::kRowBytes + ((chunk ^ G::swz_v(vrow)) << 4) + 8 * (i16 & 1);
    }
  }

  // Eight-slot ring: LDS addresses of the operand reads for the ring's two halves.  A step whose
  // ring position is known at compile time (the unrolled blocks of eight steps below) reads its
  // operands at one of these plus an immediate offset and spends no instruction on addresses.
  constexpr bool kStaticRing = kPair && kSlots == 8 && 4 * G::kSlotBytes <= 65536;
  constexpr int kHalves = kStaticRing ? 2 : 1;
  unsigned kbase[kHalves][NKA], vbase[kHalves][NB];
#pragma unroll
  for (int hf = 0; hf < kHalves; ++hf) {
#pragma unroll
    for (int i = 0; i < NKA; ++i) kbase[hf][i] = (unsigned)(size_t)lds + (unsigned)(koff[i] + hf * 4 * G::kSlotBytes);
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) vbase[hf][nb] = (unsigned)(size_t)lds + (unsigned)(voff[nb] + hf * 4 * G::kSlotBytes);
  }

  f32x16 O[QB][NB];
  float m_ref[QB], mc_ref[QB], l_run[QB];  // mc_ref = m_ref * c
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    m_ref[qb] = -INFINITY;
    mc_ref[qb] = -INFINITY;
    l_run[qb] = 0.f;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
      for (int r = 0; r < 16; ++r) O[qb][nb][r] = 0.f;
  }

  // ---- operand fetch from LDS.  Inline asm: the order and the waits are ours (the compiler
  //      would make a transposing read wait for every outstanding global->LDS load).
  // K operand of k-chunk kc for the step in the slot at byte offset `so`
  auto k_load = [&](int so, i32x4(&Kr)[NC]) __attribute__((always_inline)) {
    unsigned ka[NKA];
#pragma unroll
    for (int i = 0; i < NKA; ++i) ka[i] = kbase[0][i] + (unsigned)so;
#pragma unroll
    for (int kc = 0; kc < NC; ++kc)
      asm volatile("ds_read_b128 %0, %1" : "=v"(Kr[kc]) : "v"(ka[kc]));
  };
  auto k_wait = [&](i32x4(&Kr)[NC]) __attribute__((always_inline)) {
    if constexpr (NC == 8) {
      asm volatile("s_waitcnt lgkmcnt(0)"
                   : "+v"(Kr[0]), "+v"(Kr[1]), "+v"(Kr[2]), "+v"(Kr[3]), "+v"(Kr[4]), "+v"(Kr[5]), "+v"(Kr[6]),
                     "+v"(Kr[7]));
    } else {
      asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(Kr[0]), "+v"(Kr[1]), "+v"(Kr[2]), "+v"(Kr[3]));
    }
  };
  // V^T operand: k-slot e of half-wave hi in chunk h2 is key 16 h2 + 8 (e/4) + 4 hi + e%4 (the
  // accumulator layout of S^T), so V^T is fetched for exactly those keys: two transposing reads
  // of 4 keys each per (h2, 32-row block nb).
  auto v_load = [&](int so, s16x4(&Vr)[2][NB][2]) __attribute__((always_inline)) {
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      const unsigned va = vbase[0][nb] + (unsigned)so;
#pragma unroll
      for (int h2 = 0; h2 < 2; ++h2) {
        asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(Vr[h2][nb][0]) : "v"(va), "n"(16 * h2 * G::kRowBytes));
        asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2"
                     : "=v"(Vr[h2][nb][1])
                     : "v"(va), "n"((16 * h2 + 8) * G::kRowBytes));
      }
    }
  };
  auto v_wait = [&](s16x4(&Vr)[2][NB][2]) __attribute__((always_inline)) {
    if constexpr (NB == 4) {
      asm volatile("s_waitcnt lgkmcnt(0)"
                   : "+v"(Vr[0][0][0]), "+v"(Vr[0][0][1]), "+v"(Vr[0][1][0]), "+v"(Vr[0][1][1]), "+v"(Vr[0][2][0]),
                     "+v"(Vr[0][2][1]), "+v"(Vr[0][3][0]), "+v"(Vr[0][3][1]), "+v"(Vr[1][0][0]), "+v"(Vr[1][0][1]),
                     "+v"(Vr[1][1][0]), "+v"(Vr[1][1][1]), "+v"(Vr[1][2][0]), "+v"(Vr[1][2][1]), "+v"(Vr[1][3][0]),
                     "+v"(Vr[1][3][1]));
    } else {
      asm volatile("s_waitcnt lgkmcnt(0)"
                   : "+v"(Vr[0][0][0]), "+v"(Vr[0][0][1]), "+v"(Vr[0][1][0]), "+v"(Vr[0][1][1]), "+v"(Vr[1][0][0]),
                     "+v"(Vr[1][0][1]), "+v"(Vr[1][1][0]), "+v"(Vr[1][1][1]));
    }
  };
  // ---- matrix products
  auto s_mma = [&](const i32x4(&Kr)[NC], f32x16(&S)[QB]) __attribute__((always_inline)) {
    const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kc = 0; kc < NC; ++kc)
#pragma unroll
      for (int qb = 0; qb < QB; ++qb)
        S[qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, Kr[kc]), Qr[qb][kc],
                                                        kc == 0 ? zero : S[qb], 0, 0, 0);
  };
  // One PV product O^T[qb][nb] += V^T(h2, nb) . P^T[qb][h2]
  auto pv_one = [&](const s16x4(&Vr)[2][NB][2], const bf16x8(&P)[QB][2], int h2, int nb, int qb) __attribute__((always_inline)) {
    const bf16x8 va =
        __builtin_bit_cast(bf16x8, __builtin_shufflevector(Vr[h2][nb][0], Vr[h2][nb][1], 0, 1, 2, 3, 4, 5, 6, 7));
    O[qb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, P[qb][h2], O[qb][nb], 0, 0, 0);
  };
  auto pv_mma = [&](const s16x4(&Vr)[2][NB][2], const bf16x8(&P)[QB][2], int h2) __attribute__((always_inline)) {
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) pv_one(Vr, P, h2, nb, qb);
  };
  auto compute_s = [&](int so, f32x16(&S)[QB]) __attribute__((always_inline)) {  // unpipelined S^T of the step in slot `so`
    i32x4 Kr[NC];
    k_load(so, Kr);
    k_wait(Kr);
    s_mma(Kr, S);
  };
  auto pv = [&](int so, const bf16x8(&P)[QB][2]) __attribute__((always_inline)) {  // unpipelined O^T += V^T P^T
    s16x4 Vr[2][NB][2];
    v_load(so, Vr);
    v_wait(Vr);
    pv_mma(Vr, P, 0);
    pv_mma(Vr, P, 1);
  };
  // S^T accumulators (produced in vector registers: VGPR-form products) as plain floats
  auto s_fetch = [&](const f32x16(&S)[QB], float(&Sv)[QB][16]) __attribute__((always_inline)) {
#pragma unroll
    for (int qb = 0; qb < QB; ++qb)
#pragma unroll
      for (int r = 0; r < 16; ++r) Sv[qb][r] = S[qb][r];
  };
  // P = exp2(S c - m_ref c) as bf16 and its row sums (of the rounded values)
  auto softmax = [&](const float(&S)[QB][16], bf16x8(&P)[QB][2], float(&psum)[QB]) __attribute__((always_inline)) {
    const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      const float mc = mc_ref[qb];
      float ps = 0.f;
#pragma unroll
      for (int h2 = 0; h2 < 2; ++h2) {
        f32x8 e;
#pragma unroll
        for (int t = 0; t < 8; ++t) e[t] = __builtin_amdgcn_exp2f(fmaf(S[qb][8 * h2 + t], c, -mc));
        const bf16x8 pb = __builtin_convertvector(e, bf16x8);
        P[qb][h2] = pb;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          const bf16x2 pr = {pb[2 * t], pb[2 * t + 1]};
          ps = __builtin_amdgcn_fdot2_f32_bf16(pr, ones, ps, false);
        }
      }
      psum[qb] = ps;
    }
  };
  auto row_max = [&](const float(&S)[QB][16], int qb) __attribute__((always_inline)) {
    float mx = fmaxf(S[qb][0], S[qb][1]);
#pragma unroll
    for (int r = 2; r < 16; r += 2) mx = fmaxf(fmaxf(mx, S[qb][r]), S[qb][r + 1]);
    return half_max(mx);
  };
  auto rescale = [&](int qb, float alpha) __attribute__((always_inline)) {  // rare: O^T and l of query block qb times alpha
    l_run[qb] *= alpha;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
      for (int r = 0; r < 16; ++r) O[qb][nb][r] = O[qb][nb][r] * alpha;
  };
  // Validate the P just formed (before anything uses it).  A lane's row sum can only exceed
  // 2^8 if one of its weights does, i.e. if a score of this step exceeds the reference maximum
  // by more than 2^8/... ; then the reference is raised to the step's true maximum, the
  // accumulators are rescaled and this P is formed again.  exp2 can therefore not overflow
  // into the accumulators, and the common path pays two compares.
  auto settle = [&](const float(&S)[QB][16], bf16x8(&P)[QB][2], float(&psum)[QB]) __attribute__((always_inline)) {
    bool any = false;
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) any |= !(psum[qb] <= kLazyLimit);
    if (__builtin_expect(__builtin_amdgcn_ballot_w64(any) != 0, 0)) {  // rare: laid out off the step's straight path
      // The first P stays "used" on this path too, so that its computation is not sunk below
      // the branch (it has to overlap with the matrix products above).
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) asm volatile("" ::"v"(P[qb][0]), "v"(P[qb][1]), "v"(psum[qb]));
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) {
        const float mx = row_max(S, qb);
        const float m_new = fmaxf(m_ref[qb], mx);
        const float alpha = __builtin_amdgcn_exp2f((m_ref[qb] - m_new) * c);
        m_ref[qb] = m_new;
        mc_ref[qb] = m_new * c;
        rescale(qb, alpha);
      }
      softmax(S, P, psum);
    }
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) l_run[qb] += psum[qb];
  };

  // ring offsets of steps j-1, j, j+1, j+2
  int so_m1 = 0, so_0 = 0, so_p1 = G::kSlotBytes, so_p2 = 2 * G::kSlotBytes;
  auto advance = [&]() __attribute__((always_inline)) {
    so_m1 = so_0;
    so_0 = so_p1;
    so_p1 = so_p2;
    so_p2 = next_slot(so_p2);
  };

  // Element mask of step j: the lane's query (row tw0 + 32 qb + col of the segment) sees the keys
  // of a span-1 step up to its own row and the keys of a span-0 step up to the span's end.
  auto mask_step = [&](float(&S)[QB][16], int j) __attribute__((always_inline)) {
    const bool s1 = j >= nst0;
    const int j0 = (s1 ? j - nst0 : j) * kStepKeys;
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      int t = tw0 + 32 * qb + col;
      t = t < last_row ? t : last_row;
      const int lim = (s1 ? t + 1 : w.n0) - j0 - 4 * hi;  // first invisible key, relative to the lane's keys
#pragma unroll
      for (int r = 0; r < 16; ++r)
        if (8 * (r >> 2) + (r & 3) >= lim) S[qb][r] = -INFINITY;
    }
  };
  auto sync_step_hot = [&](auto plain) __attribute__((always_inline)) {
    SEGATTN_VMCNT(kAhead * 2 * LPW);
    __builtin_amdgcn_s_barrier();
    issue_loads();
    if constexpr (kPair) {
      if constexpr (decltype(plain)::value) loader_advance_plain();
      else loader_advance();
      issue_loads();
    }
  };
  // One pipelined step j >= 1.  On entry Kr holds the K operands of step j+1, Sc is S^T of step
  // j and Pp is P of step j-1.  The step forms S^T(j+1) -> Sn, adds PV of step j-1, turns Sc
  // into Pc, runs the step's sync in the middle and leaves the K operands of step j+2 in Kr.
  // Beyond the last step the operands are those of a step fetched again: finite and unused.
  // MASKED: keys of step j with in-span index >= the lane's limit are invisible (the diagonal
  // of the query's own segment, the ragged end of a span).
  // Laid out by hand as 2*NC + 4*NB slots of one matrix product
  // each; whatever else the step has to do is spread over the slots so that it issues in the
  // shadow of the products (about six vector instructions fit under a 32x32x16 MFMA).  The
  // sync is branch-free: exactly one step of loads stays in flight and the loads issued are a
  // full step of the current span.
  //   slots 0 .. 2NC-1        S^T(j+1) products; all V^T reads; exp2 of pair i in slot 2i
  //   slots 2NC .. 2NC+2NB-1  PV(j-1), first 16 keys
  //   (sync, then the K reads of step j+2, two per slot)
  //   slots .. end            PV(j-1), last 16 keys
  //   odd slots               convert pair i to bf16 and add it to the row sum
  // ring_pos: -1, or (as a compile-time tag) the ring slot of step j-1, from which the slots of the
  // step's operand reads follow: V^T of step j-1 there, K of step j+2 three slots on.
  auto hot_step = [&](auto masked, auto plain, auto syncs, auto ring_pos, int j, i32x4(&Kr)[NC], float(&Sc)[QB][16],
                      float(&Sn)[QB][16], const bf16x8(&Pp)[QB][2], bf16x8(&Pc)[QB][2]) __attribute__((always_inline)) {
    if constexpr (decltype(masked)::value) mask_step(Sc, j);
    constexpr int RP = decltype(ring_pos)::value;
    constexpr bool kFixed = RP >= 0;
    constexpr int vslot = kFixed ? RP : 0, kslot = kFixed ? (RP + 3) % 8 : 0;
    constexpr int vimm = (vslot % 4) * G::kSlotBytes, kimm = (kslot % 4) * G::kSlotBytes;
    static_assert(!kFixed || kStaticRing, "fixed ring positions need the eight-slot ring");
    constexpr int NS = QB * NC, NP = QB * NB;  // slots of the S^T product / of half a PV product
    constexpr int NSLOT = NS + 2 * NP;
    constexpr int NE = 16 * QB;                // softmax elements per lane and step
    constexpr int EPS = NE / NSLOT;            // of them per slot
    static_assert(EPS * NSLOT == NE && (EPS == 1 || EPS == 2), "slot layout");
    const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
    const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    float psum[QB] = {};
    s16x4 Vr[2][NB][2];
    f32x16 Sacc[QB];
    int Pw[QB][8];  // P of the current step as 32-bit words: word 4 h2 + t of Pw[qb] = elements 8 h2 + 2t, +1
    float ev[NE];   // exp2 results on their way to the bf16 pairs (a few live at a time)
    unsigned va[NB], ka[NKA];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
      va[nb] = kFixed ? vbase[kFixed ? vslot / 4 : 0][nb] : vbase[0][nb] + (unsigned)so_m1;
#pragma unroll
    for (int i = 0; i < NKA; ++i)
      ka[i] = kFixed ? kbase[kFixed ? kslot / 4 : 0][i] : kbase[0][i] + (unsigned)so_p2;
    // vector-ALU work of one slot: exp2 of EPS elements, and half of the conversion / row-sum
    // work of an earlier pair, so that every slot carries the same four issue slots
    auto valu_chunk = [&](int slot) __attribute__((always_inline)) {
#pragma unroll
      for (int u = 0; u < EPS; ++u) {
        const int e = EPS * slot + u, qb = e / 16, r = e % 16;
        ev[e] = __builtin_amdgcn_exp2f(fmaf(Sc[qb][r], c, -mc_ref[qb]));
      }
      // pair index handled now: its two exp2 were issued at least one slot ago
      const int first_pair = (EPS == 1) ? (slot / 2 - 1) : (slot - 1);
      if (first_pair >= 0) {
        const int i = first_pair, qb = i / 8, w8 = i % 8;
        typedef float f32x2 __attribute__((ext_vector_type(2)));
        if (EPS == 2 || slot % 2 == 0) {
          const f32x2 ee = {ev[2 * i], ev[2 * i + 1]};
          Pw[qb][w8] = __builtin_bit_cast(int, __builtin_convertvector(ee, bf16x2));
        }
        if (EPS == 2 || slot % 2 == 1) {
          // the first pair starts the row sum: the three-operand form with a zero addend (the compiler's
          // choice is a move of zero and the accumulating two-operand form)
          if (w8 == 0)
            asm("v_dot2_f32_bf16 %0, %1, %2, 0" : "=v"(psum[qb]) : "v"(Pw[qb][w8]), "s"(0x3f803f80));
          else
            psum[qb] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, Pw[qb][w8]), ones, psum[qb], false);
        }
      }
    };
    // transposing V^T reads per slot: one more than an even spread needs, so that the last reads
    // have two product slots to land before the wait in front of the sync (measured: +1.7 %;
    // denser bursts lose)
    constexpr int VPS = (4 * NB + NS - 1) / NS + 1;
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int slot = 0; slot < NSLOT; ++slot) {
      // ---- the slot's matrix product
      if (slot < NS) {
        const int kc = slot / QB, qb = slot % QB;
        Sacc[qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, Kr[kc]), Qr[qb][kc],
                                                           kc == 0 ? zero : Sacc[qb], 0, 0, 0);
      } else {
        const int t = slot - NS, h2 = t / NP, nb = (t % NP) / QB, qb = t % QB;
        pv_one(Vr, Pp, h2, nb, qb);
      }
      __builtin_amdgcn_sched_barrier(0);
      // ---- V^T reads (h2-major), spread over the S^T slots so that the four waves of the
      //      workgroup, which run in lockstep, do not all hit the LDS in one burst
      {
#pragma unroll
        for (int u = 0; u < VPS; ++u) {
          const int idx = VPS * slot + u;  // 0 .. 4 NB - 1: (h2, nb, half)
          if (idx < 4 * NB) {
            const int h2 = idx / (2 * NB), nb = (idx / 2) % NB, half = idx % 2;
            if (half == 0)
              asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2"
                           : "=v"(Vr[h2][nb][0]) : "v"(va[nb]), "n"(16 * h2 * G::kRowBytes + vimm));
            else
              asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2"
                           : "=v"(Vr[h2][nb][1]) : "v"(va[nb]), "n"((16 * h2 + 8) * G::kRowBytes + vimm));
          }
        }
      }
      // ---- after the S^T slots: V^T has arrived; sync; then the K reads of step j+2, one per slot
      constexpr int kSyncSlot = NS - 1;
      if (slot == kSyncSlot) {
        v_wait(Vr);
        if constexpr (std::is_same<decltype(syncs), bool>::value) {
          if (syncs) sync_step_hot(plain);  // decided at run time (uniform): the general step
        } else if constexpr (decltype(syncs)::value) {
          sync_step_hot(plain);
        }
      }
      if (slot > kSyncSlot && slot - kSyncSlot - 1 < NC) {
        const int kc = slot - kSyncSlot - 1;
        asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(Kr[kc]) : "v"(ka[kc]), "n"(kimm));
      }
      valu_chunk(slot);
      __builtin_amdgcn_sched_barrier(0);
    }
    {  // the last pair(s)
      typedef float f32x2 __attribute__((ext_vector_type(2)));
      const int qb = QB - 1;
      const f32x2 ee = {ev[NE - 2], ev[NE - 1]};
      Pw[qb][7] = __builtin_bit_cast(int, __builtin_convertvector(ee, bf16x2));
      psum[qb] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, Pw[qb][7]), ones, psum[qb], false);
    }
#pragma unroll
    for (int qb = 0; qb < QB; ++qb)
#pragma unroll
      for (int h2 = 0; h2 < 2; ++h2) {
        const i32x4 w4 = {Pw[qb][4 * h2], Pw[qb][4 * h2 + 1], Pw[qb][4 * h2 + 2], Pw[qb][4 * h2 + 3]};
        Pc[qb][h2] = __builtin_bit_cast(bf16x8, w4);
      }
    s_fetch(Sacc, Sn);
    // (All K reads are waited for here, not one by one in front of their products in the next
    // step: until the wait the compiler believes the registers already hold the data, and any
    // move it placed in between -- a spill, a copy at the loop edge -- would carry stale values.)
    k_wait(Kr);
    settle(Sc, Pc, psum);
    if constexpr (std::is_same<decltype(syncs), bool>::value) {
      if (syncs) loader_advance();
    } else if constexpr (decltype(syncs)::value) {
      if constexpr (decltype(plain)::value) loader_advance_plain();
      else loader_advance();
    }
  };
  // =========================== main sequence ===========================
  sync_step();
  loader_advance();
  float Sa[QB][16] = {}, Sb[QB][16] = {};
  bf16x8 Pa[QB][2] = {}, Pb[QB][2] = {};
  i32x4 Kr[NC] = {};
  {  // step 0 without overlap: exact maximum as the first reference (every query sees key 0 of
     // its first step)
    float psum[QB];
    f32x16 Sacc[QB];
    compute_s(so_0, Sacc);
    s_fetch(Sacc, Sa);
    if (f == 0) mask_step(Sa, 0);
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      float mx = Sa[qb][0];
#pragma unroll
      for (int r = 1; r < 16; ++r) mx = fmaxf(mx, Sa[qb][r]);
      m_ref[qb] = half_max(mx);
      mc_ref[qb] = m_ref[qb] * c;
    }
    softmax(Sa, Pb, psum);
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) l_run[qb] = psum[qb];
    compute_s(so_p1, Sacc);
    s_fetch(Sacc, Sa);
    k_load(so_p2, Kr);  // K operands of step 2 for the product formed in step 1
    k_wait(Kr);
  }
  int j = 1;
  advance();
  constexpr std::true_type yes{};
  constexpr std::false_type no{};
  // here and at the top of every iteration below: Sa = S^T(j), Pb = P(j-1), Kr = K operands of j+1
  constexpr std::integral_constant<int, -1> anywhere{};
  while (j < n_act) {
    // Blocks of eight unmasked steps at fixed ring positions (eight-slot ring): step j sits in slot
    // j % 8 for the whole item, so from j = 1 (mod 8) on -- where the sequence starts -- the eight
    // steps of a block read their operands at compile-time offsets; the slot variables return to
    // where they were after eight steps and are left alone.
    if constexpr (kStaticRing) {
      while ((j & 7) == 1 && j + 7 < f && ld_js + 8 < ld_full_end) {
        hot_step(no, yes, no, std::integral_constant<int, 0>{}, j, Kr, Sa, Sb, Pb, Pa);
        hot_step(no, yes, yes, std::integral_constant<int, 1>{}, j + 1, Kr, Sb, Sa, Pa, Pb);
        hot_step(no, yes, no, std::integral_constant<int, 2>{}, j + 2, Kr, Sa, Sb, Pb, Pa);
        hot_step(no, yes, yes, std::integral_constant<int, 3>{}, j + 3, Kr, Sb, Sa, Pa, Pb);
        hot_step(no, yes, no, std::integral_constant<int, 4>{}, j + 4, Kr, Sa, Sb, Pb, Pa);
        hot_step(no, yes, yes, std::integral_constant<int, 5>{}, j + 5, Kr, Sb, Sa, Pa, Pb);
        hot_step(no, yes, no, std::integral_constant<int, 6>{}, j + 6, Kr, Sa, Sb, Pb, Pa);
        hot_step(no, yes, yes, std::integral_constant<int, 7>{}, j + 7, Kr, Sb, Sa, Pa, Pb);
        j += 8;
      }
      if (j >= n_act) break;
    }
    // pairs of steps that need no mask while the loader stays inside plain full steps of its span
    // (with the pair sync a pair is an odd step, which meets nobody, and the even step after it)
    if (!kPair || (j & 1)) {
      while (j + 1 < f && ld_js + 2 < ld_full_end) {
        if constexpr (kPair) hot_step(no, yes, no, anywhere, j, Kr, Sa, Sb, Pb, Pa);
        else hot_step(no, yes, yes, anywhere, j, Kr, Sa, Sb, Pb, Pa);
        advance();
        hot_step(no, yes, yes, anywhere, j + 1, Kr, Sb, Sa, Pa, Pb);
        advance();
        j += 2;
      }
      if (j >= n_act) break;
    }
    // any other step (the loader is at a span switch, a ragged step or its last step, or the
    // step needs a mask): the masked step with the loader's general advance; a mask that hides
    // nothing is harmless.  Its results move back into (Sa, Pb) so that the roles stay fixed
    // (choosing between the two register sets at run time would put them in memory).
    if constexpr (kPair) hot_step(yes, no, !(j & 1), anywhere, j, Kr, Sa, Sb, Pb, Pa);
    else hot_step(yes, no, yes, anywhere, j, Kr, Sa, Sb, Pb, Pa);
    advance();
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
#pragma unroll
      for (int r = 0; r < 16; ++r) Sa[qb][r] = Sb[qb][r];
      Pb[qb][0] = Pa[qb][0];
      Pb[qb][1] = Pa[qb][1];
    }
    ++j;
  }
  // so_m1 is the slot of the wave's last step, whose P waits in Pb
  pv(so_m1, Pb);
  // steps that only other waves of the workgroup need (a workgroup with several 32-row blocks per
  // head ends on the diagonal of its last block): keep loading and meeting at the barriers
  for (; j < n; ++j) {
    if (!kPair || !(j & 1)) {
      sync_step();
      loader_advance();
    }
  }
  SEGATTN_VMCNT(0);  // the loader's surplus loads have landed: the ring may be reused
  unsigned ticket = 0;
  if (next_from && tid == 0) ticket = atomicAdd(next_from, 1u);

  // ---- epilogue: normalise, write LSE, and write O through LDS so that every store
  // instruction covers whole 16-byte pieces of contiguous output rows.  A lane holds four
  // consecutive d of one query row per accumulator quad; it drops them into the wave's own
  // [32 rows][D] staging block (rows padded by 8 bytes against bank conflicts), and the wave
  // reads the block back row-major.
  __syncthreads();  // every wave is past its last read of the K/V ring
  const bool wide = w.wide;
  const int es = wide ? 4 : 2;                 // bytes per output element
  const int row_bytes = D * es + 8;
  unsigned char *stage = smem + wave * (32 * (D * es + 8));
  const int lanes_per_row = D * es / 16;       // 16-byte pieces per output row
  const int rows_per_pass = 64 / lanes_per_row;
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const int t = tw0 + 32 * qb + col;
    const float l = half_sum(l_run[qb]);
    const float inv = 1.f / l;
    if (hi == 0 && t <= last_row) w.lse[(long long)ohead * w.lse_head_stride + t] = m_ref[qb] * p.scale + __logf(l);
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
      for (int rg = 0; rg < 4; ++rg) {
        const int d = 32 * nb + 8 * rg + 4 * hi;
        const f32x4 o = {O[qb][nb][4 * rg + 0] * inv, O[qb][nb][4 * rg + 1] * inv,
                         O[qb][nb][4 * rg + 2] * inv, O[qb][nb][4 * rg + 3] * inv};
        unsigned char *dst = stage + col * row_bytes + d * es;
        if (wide) {
          *(uint2 *)dst = uint2{__float_as_uint(o[0]), __float_as_uint(o[1])};
          *(uint2 *)(dst + 8) = uint2{__float_as_uint(o[2]), __float_as_uint(o[3])};
        } else {
          *(uint2 *)dst = __builtin_bit_cast(uint2, __builtin_convertvector(o, bf16x4));
        }
      }
    __syncthreads();
    const int piece = lane % lanes_per_row;
    for (int r = lane / lanes_per_row; r < 32; r += rows_per_pass) {
      const int tr = tw0 + 32 * qb + r;
      if (tr > last_row) break;
      const unsigned char *src = stage + r * row_bytes + piece * 16;
      const uint2 a0 = *(const uint2 *)src, a1 = *(const uint2 *)(src + 8);
      unsigned char *gdst = (unsigned char *)w.out + (((long long)tr * w.out_heads + ohead) * D) * es + piece * 16;
      *(uint4 *)gdst = uint4{a0.x, a0.y, a1.x, a1.y};
    }
    __syncthreads();
  }
  return ticket;
}

// One work item per workgroup, the block index (PrefillArgs::queue == nullptr), or a resident
// grid -- as many workgroups as fit the chip -- that takes item after item from eight queues.
//
// The hardware deals the workgroups of a launch to the 8 XCDs by index (XCD = index % 8) and every
// XCD works through its share at its own pace.  Under this kernel the XCDs of one part differ by
// 4-8 % in speed (timestamps per workgroup: the same work on each, every CU of an XCD finishing
// together, the XCDs up to 6 % apart), so with a fixed share each the launch ends with most of
// the chip waiting for the slowest XCD; and between two workgroups a CU idles 4-6 us.  In the
// queued form queue x holds the items x, x+8, ... that XCD x would have been dealt, in the same
// order, and a workgroup on XCD x takes from queue x first: the L2 locality of the mapping in
// resolve() is untouched.  Once its own queue is empty a workgroup takes from the queue with the
// most items left, so a fast XCD goes on with the slowest one's items; when all eight are empty
// it leaves.  Nothing waits for another workgroup.  The ticket for the next round is drawn while
// the output of this one is being written (prefill_mfma_item), so the round trip to the counter
// is hidden.  Each queue's counter has a 128-byte line of its own; a one-wave kernel in front of
// the launch clears them.
template <int D, int HS, int QB, int NW>
__global__ __launch_bounds__(64 * NW, 8 / (NW * QB)) void prefill_mfma_kernel(const Problem p_arg, const PrefillArgs a_arg) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  // take_item's hand-over word lives at the start of the ring, which is idle between two items (a
  // static variable of its own would be the four bytes by which two four-wave workgroups, 80 KB of
  // ring each, no longer fit the 160 KB of a CU)
  int *const claim = (int *)smem;
  constexpr unsigned kArgsAt = (sizeof(Problem) + alignof(PrefillArgs) - 1) / alignof(PrefillArgs) * alignof(PrefillArgs);
  unsigned ticket = 0;  // thread 0: position drawn from the own queue for this round
  bool drawn = false;   // ... by the previous round already
  for (;;) {
    // The arguments are read through a pointer the compiler cannot see through, once per round
    // (and the item reads its thread index the same way): read as plain kernel arguments and
    // built-ins they are loop invariants, everything derived from them is hoisted out of the
    // loop and stays in registers for all of it, and this kernel has none to spare.
    const __attribute__((address_space(4))) unsigned char *ka =
        (const __attribute__((address_space(4))) unsigned char *)__builtin_amdgcn_kernarg_segment_ptr();
    asm volatile("" : "+s"(ka));
    const Problem &p = *(const Problem *)ka;
    const PrefillArgs &a = *(const PrefillArgs *)(ka + kArgsAt);
    int bid = (int)blockIdx.x;
    const bool queued = a.queue != nullptr;
    unsigned *const own = queued ? a.queue + kQueueStride * ((int)blockIdx.x & 7) : nullptr;
    if (queued) {
      bid = take_item(a.queue, a.grid_items, drawn, ticket, claim);
      if (bid < 0) return;
    }
    ticket = prefill_mfma_item<D, HS, QB, NW>(p, a, bid, smem, own);
    drawn = true;
    if (!queued) return;
  }
}

// Clears a set of queue counters (launched in front of every queued launch, on its stream).
__global__ void item_queue_reset_kernel(unsigned *queue) {
  if (threadIdx.x < 8) queue[kQueueStride * threadIdx.x] = 0;
}

std::mutex &item_queue_launch_mutex() {
  static std::mutex mu;
  return mu;
}

hipError_t item_queue_reset(unsigned *queue, hipStream_t st) {
  hipLaunchKernelGGL(item_queue_reset_kernel, dim3(1), dim3(64), 0, st, queue);
  return hipGetLastError();
}

// =============================================================================================
// split prefix (segment-by-segment prefill): merge the pieces
// =============================================================================================
// Every piece of a PAST head's keys left a normalised fp32 output row and its LSE in the
// workspace; softmax over the union is the LSE-weighted mean of the pieces (the same identity the
// decode path and a sharded prefix use).  32 lanes per (sequence, row, head), D/32 channels each.
template <int D>
__global__ __launch_bounds__(256) void prefill_part_combine_kernel(const Problem p, const PrefillArgs a) {
  constexpr int CPL = D / 32;  // channels per lane
  const int ph = p.n_past * p.g;
  const long long m = a.n_rows;
  const long long item = (long long)blockIdx.x * 8 + (threadIdx.x >> 5);
  if (item >= (long long)p.B * m * ph) return;
  const int lane = threadIdx.x & 31;
  const int hc = (int)(item % ph);
  const long long row = (item / ph) % m;
  const int b = (int)(item / ((long long)ph * m));
  const int head = p.order[hc / p.g] * p.g + hc % p.g;
  float mx = -INFINITY;
  for (int pt = 0; pt < a.parts; ++pt)
    mx = fmaxf(mx, a.part_lse[(((long long)b * a.parts + pt) * ph + hc) * m + row]);
  float sum = 0.f, acc[CPL];
#pragma unroll
  for (int e = 0; e < CPL; ++e) acc[e] = 0.f;
  for (int pt = 0; pt < a.parts; ++pt) {
    const float wgt = __expf(a.part_lse[(((long long)b * a.parts + pt) * ph + hc) * m + row] - mx);
    const float *src = a.part_out + ((((long long)b * a.parts + pt) * m + row) * ph + hc) * D + lane * CPL;
    sum += wgt;
#pragma unroll
    for (int e = 0; e < CPL; ++e) acc[e] = fmaf(wgt, src[e], acc[e]);
  }
  const float inv = 1.f / sum;
  const long long o = (((long long)b * m + row) * p.Hq + head) * D + lane * CPL;
#pragma unroll
  for (int e = 0; e < CPL; ++e) {
    if (p.out_fp32) ((float *)a.out)[o + e] = acc[e] * inv;
    else ((__bf16 *)a.out)[o + e] = (__bf16)(acc[e] * inv);
  }
  if (lane == 0) a.lse[((long long)b * p.Hq + head) * m + row] = mx + __logf(sum);
}

// =============================================================================================
// launch
// =============================================================================================
hipError_t launch_prefill_fp32(const Problem &p, const PrefillArgs &a, long long grid, hipStream_t st);

static int heads_per_wg(const Problem &p) { return (p.g % 4 == 0) ? 4 : (p.g % 2 == 0) ? 2 : 1; }

// ---- counters of the queued form of the kernel
// Eight counters per set, each on a 128-byte line of its own.  Launches on one stream run one
// after the other and share a set; launches on different streams may overlap, so every (device, stream) pair that asks gets a
// set of its own, for as long as the process lives.  When the sets are used up, and for a stream
// that is being captured (the graph may later be replayed on any stream, next to anything), the
// launch falls back to one workgroup per item, which needs no counters.
static int device_cus();

constexpr int kQueueSets = 64;
constexpr int kQueueDevices = 16;
static __device__ unsigned g_queue_sets[kQueueSets][8 * kQueueStride];

unsigned *item_queue_for(hipStream_t st) {
  struct Owner {
    int dev;
    hipStream_t st;
  };
  static std::mutex mu;
  static Owner owners[kQueueSets];
  static int n_owners = 0;
  static unsigned *base[kQueueDevices] = {};
  hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
  if (hipStreamIsCapturing(st, &cs) != hipSuccess) {
    (void)hipGetLastError();
    return nullptr;
  }
  if (cs != hipStreamCaptureStatusNone) return nullptr;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kQueueDevices) return nullptr;
  std::lock_guard<std::mutex> lock(mu);
  if (!base[dev]) {
    void *ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(g_queue_sets)) != hipSuccess || !ptr) {
      (void)hipGetLastError();
      return nullptr;
    }
    base[dev] = (unsigned *)ptr;
  }
  int set = -1;
  for (int i = 0; i < n_owners; ++i)
    if (owners[i].dev == dev && owners[i].st == st) set = i;
  if (set < 0) {
    if (n_owners == kQueueSets) return nullptr;
    owners[n_owners] = Owner{dev, st};
    set = n_owners++;
  }
  return base[dev] + 8 * kQueueStride * set;
}

template <int D, int HS, int QB, int NW>
static hipError_t launch_mfma(const Problem &p, const PrefillArgs &a_in, long long grid, hipStream_t st) {
  constexpr int ring = ring_slots(NW, QB) * StepGeom<D>::kSlotBytes;
  constexpr int epilogue = NW * 32 * (D * 4 + 8);  // fp32 output staging, one block per wave
  constexpr int lds = ring > epilogue ? ring : epilogue;
  auto kern = prefill_mfma_kernel<D, HS, QB, NW>;
  // First launch of this instantiation: allow the kernel its LDS, ask how many workgroups the chip
  // holds.  Both steps give the same result whoever does them, so host threads racing through
  // their first call simply do them twice; `ready` is set only after the attribute is in place.
  static std::atomic<bool> ready{false};
  static ResidentCount resident_count;
  if (!ready.load(std::memory_order_acquire)) {
    hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (e != hipSuccess) return e;
    ready.store(true, std::memory_order_release);
  }
  const int resident = resident_count.get((const void *)kern, 64 * NW, lds);  // 0: unknown, no queues
  PrefillArgs a = a_in;
  a.grid_items = (int)grid;
  a.queue = nullptr;
  long long launch = item_queue_grid(p, grid, resident);
  if (launch != grid || (p.tune_queue >= 2 && grid > 1 && resident > 0)) {
    a.queue = item_queue_for(st);
    if (!a.queue) launch = grid;
  }
  if (!a.queue) {
    hipLaunchKernelGGL(kern, dim3((unsigned)launch), dim3(64 * NW), lds, st, p, a);
    return hipGetLastError();
  }
  // reset and launch go into the stream back to back, also when several host threads use it
  std::lock_guard<std::mutex> pair(item_queue_launch_mutex());
  hipError_t e = item_queue_reset(a.queue, st);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, dim3((unsigned)launch), dim3(64 * NW), lds, st, p, a);
  return hipGetLastError();
}

// Stride of the group shuffle in resolve(): the smallest number >= groups/8 that is coprime to
// the number of groups.
int prefill_pair_stride(long long groups) {
  if (groups <= 1) return 1;
  auto gcd = [](long long x, long long y) {
    while (y) {
      const long long t = x % y;
      x = y;
      y = t;
    }
    return x;
  };
  long long s = groups / 8 > 0 ? groups / 8 : 1;
  while (gcd(s, groups) != 1) ++s;
  return (int)s;
}

// Waves per workgroup for head_dim 128 (each wave owns one head x 32 query rows; D = 64 always
// runs four waves, whose step of 32 keys is only four 1 KB loads per tensor).  Eight waves -- 64 rows per head, one workgroup per CU, two waves
// per SIMD -- move half as many K/V bytes per query row and are the choice whenever there is
// enough work to fill the chip.  Four waves -- 32 rows per head, two workgroups fit a CU -- double
// the number of workgroups: right when the long (PAST) workgroups of a launch would otherwise
// leave CUs idle, which is the case for a segment-by-segment prefill (one segment has 64-row
// blocks for only half of the CUs, and they carry nearly all of the work).
// segattn_config.prefill_waves overrides the choice (the tests run both shapes on small inputs).
static int waves_d128(const Problem &p, const PrefillArgs &a, int hs) {
  if (p.tune_waves == 4 || p.tune_waves == 8) return p.tune_waves;
  const int n_cu = device_cus();
  const long long seg_rows = a.n_rows < p.S ? a.n_rows : p.S;
  const int rows8 = (8 / hs) * 32;
  const long long blocks8 = (long long)a.n_seg * ((seg_rows + rows8 - 1) / rows8);
  // PAST heads carry the long key ranges unless they attend to a retrieved prefix of bounded size
  const bool long_past = p.n_past > 0 && !(a.cache != nullptr && a.geom.ret_cap > 0) && a.ret_k == nullptr;
  const long long heads = (long long)p.B * (long_past ? p.n_past : p.Hkv) * (p.g / hs);
  return heads * blocks8 < n_cu ? 4 : 8;
}

static int device_cus() {
  static const int n_cu = [] {
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
      cus = 256;
    return cus;
  }();
  return n_cu;
}

// Segment-by-segment prefill: pieces to cut every PAST head's prefix into.  One segment has few
// query blocks, and the ones of the PAST heads carry nearly all the work: with one workgroup per
// block the launch takes as long as its longest workgroup while most CUs idle.  Cut so that the
// long workgroups are about as many as the CUs (eight-wave workgroups, one per CU), every piece
// keeping at least 1024 rows.
static int prefix_parts(const Problem &p, const PrefillArgs &a, int hs) {
  if (a.cache == nullptr || a.geom.part_max < 2 || p.n_past == 0 || a.geom.ret_cap > 0 || p.D != 128) return 1;
  if (p.tune_waves != 0) return 1;  // a forced workgroup shape runs unsplit
  const int rows8 = (8 / hs) * 32;
  const long long long_wgs = (long long)p.B * p.n_past * (p.g / hs) * ((a.n_rows + rows8 - 1) / rows8);
  long long parts = device_cus() / long_wgs;
  if (parts > a.geom.part_max) parts = a.geom.part_max;
  if (parts > a.min_past_prefix / 1024) parts = a.min_past_prefix / 1024;
  return parts < 2 ? 1 : (int)parts;
}

hipError_t launch_prefill(const Problem &p, const PrefillArgs &a_in, hipStream_t st) {
  const bool fp32 = p.fp32_math != 0;
  const int hs = fp32 ? 1 : heads_per_wg(p);
  PrefillArgs a = a_in;
  a.parts = fp32 ? 1 : prefix_parts(p, a, hs);
  const int nw = p.D == 128 ? (a.parts > 1 ? 8 : waves_d128(p, a_in, hs)) : 4;
  const int rows = fp32 ? 64 : (p.D == 128 ? (nw / hs) * 32 : (4 / hs) * 32);
  const long long seg_rows = a.n_rows < p.S ? a.n_rows : p.S;
  a.q_blocks_per_seg = (int)((seg_rows + rows - 1) / rows);
  const long long per_head = (long long)p.B * (p.g / hs) * a.n_seg * a.q_blocks_per_seg;
  const long long grid = per_head * ((long long)p.n_past * a.parts + (p.Hkv - p.n_past));
  if (grid <= 0 || grid > 0x7fffffffLL) return hipErrorInvalidValue;
  const int n_first = ((a.cache != nullptr && a.geom.ret_cap > 0) || a.ret_k != nullptr) ? 0 : p.n_past;  // as in resolve()
  const long long groups = (long long)p.B * (p.Hkv - n_first) * (p.g / hs) * a.n_seg;
  a.pair_stride = prefill_pair_stride(groups);
  // Interleaved sub-groups per group so that the XCDs' ranges are whole (sub-)groups: see resolve().
  // Only for groups whose K/V rows (segment + tail) exceed an XCD's 4 MB L2 anyway: sub-groups put
  // a head on several XCDs, and for a group that fits one L2 keeping it there is worth more than
  // the even split (measured: segment-by-segment prefill with S = 4096 is 1.7 % slower with them,
  // a 16K single-segment causal launch 54 % faster).
  a.sub_groups = 1;
  if (groups > 0 && (long long)(p.S + p.T) * p.D * 4 > (4ll << 20)) {
    int d = 8;  // the smallest power of two with groups * d a multiple of 8
    for (int c = 1; c <= 8; c *= 2)
      if ((groups * c) % 8 == 0) {
        d = c;
        break;
      }
    if (a.q_blocks_per_seg % d == 0) a.sub_groups = d;
  }
  if (a.parts > 1) {
    a.part_out = (float *)(a.cache + a.geom.part_off);
    a.part_lse = a.part_out + (long long)p.B * a.parts * a.n_rows * p.n_past * p.g * p.D;
  }
  prepare_resolve_divs(p, a, hs, grid);
  if (fp32) return launch_prefill_fp32(p, a, grid, st);
  hipError_t e;
  if (p.D == 128) {
    if (nw == 8) {
      if (hs == 4) e = launch_mfma<128, 4, 1, 8>(p, a, grid, st);
      else if (hs == 2) e = launch_mfma<128, 2, 1, 8>(p, a, grid, st);
      else e = launch_mfma<128, 1, 1, 8>(p, a, grid, st);
    } else {
      if (hs == 4) e = launch_mfma<128, 4, 1, 4>(p, a, grid, st);
      else if (hs == 2) e = launch_mfma<128, 2, 1, 4>(p, a, grid, st);
      else e = launch_mfma<128, 1, 1, 4>(p, a, grid, st);
    }
  } else {
    if (hs == 4) e = launch_mfma<64, 4, 1, 4>(p, a, grid, st);
    else if (hs == 2) e = launch_mfma<64, 2, 1, 4>(p, a, grid, st);
    else e = launch_mfma<64, 1, 1, 4>(p, a, grid, st);
  }
  if (e != hipSuccess || a.parts < 2) return e;
  const long long items = (long long)p.B * a.n_rows * p.n_past * p.g;
  hipLaunchKernelGGL(prefill_part_combine_kernel<128>, dim3((unsigned)((items + 7) / 8)), dim3(256), 0, st, p, a);
  return hipGetLastError();
}

}  // namespace segattn
