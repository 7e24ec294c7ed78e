// bf16 MFMA prefill kernel of libsegattn: segment-level causal attention (Eq. 12 with the
// per-head context of Eq. 13, Appendix C) for gfx950.
//
// Workgroup = 4 waves, one wave per SIMD, up to 512 registers per lane.  HS query heads of one
// GQA group share the staged K/V rows; each wave owns one head and 64 consecutive query rows
// (two 32-column MFMA blocks).  Keys are consumed in steps of 32:
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
// of 5 step slots, three steps ahead of their use; the 16-byte chunks of a row are XOR-
// swizzled by the loading lanes so that both the row-wise K reads and the transposing V reads
// are free of bank conflicts.  Steps that need an element mask (the diagonal of the query's
// own segment, the ragged end of a span) take a plain unpipelined path; steps wholly outside
// a wave's visible range are skipped.
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
#define LDS_AS __attribute__((address_space(3)))
#define GLB_AS __attribute__((address_space(1)))

constexpr int kStepKeys = 32;
constexpr int kSlots = 5;
constexpr float kLazyLog2 = 8.f;  // rescale only when a step's maximum exceeds the reference by 2^8

template <int D>
struct StepGeom {
  static constexpr int kRowBytes = 2 * D;
  static constexpr int kChunks = D / 8;                        // 16-byte chunks per row
  static constexpr int kTensorBytes = kStepKeys * kRowBytes;   // K (or V) rows of one step
  static constexpr int kSlotBytes = 2 * kTensorBytes;
  static constexpr int kInstr = kTensorBytes / 1024;           // wave-wide 1 KB loads per tensor
  static constexpr int kInstrPerWave = kInstr / 4;
  static constexpr int kRowsPerInstr = 1024 / kRowBytes;
  static constexpr int kRowsPer256 = 256 / kRowBytes;          // rows sharing one 64-bank window
  __device__ static constexpr int swz_k(int row) { return (row / kRowsPer256) % kChunks; }
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

template <int D, int HS>
__global__ __launch_bounds__(256, 1) void prefill_mfma_kernel(const Problem p, const PrefillArgs a) {
  using G = StepGeom<D>;
  constexpr int QB = 2;             // 32-query blocks per wave
  constexpr int RW = 32 * QB;       // query rows per wave
  constexpr int BQ = (4 / HS) * RW; // query rows per workgroup
  constexpr int NC = D / 16;        // k-chunks of the QK^T product
  constexpr int NB = D / 32;        // 32-row blocks of O^T
  constexpr int LPW = G::kInstrPerWave;
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];

  const WorkItem w = resolve(p, a, blockIdx.x, BQ, HS);
  if (!w.valid) return;

  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
  const int hi = lane >> 5, col = lane & 31;
  const int i16 = lane & 15, g16 = (lane >> 4) & 1;
  const int head = w.kv * p.g + w.hsub * HS + (wave % HS);
  const int tw0 = w.t0 + (wave / HS) * RW;  // first query row of this wave
  const int last_row = w.n1 - 1;
  const float c = p.scale_log2e;
  const float tau = kLazyLog2 / c;

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
  int j_active_end;  // steps at or beyond this one start after the wave's last query
  {
    const int last_q = tw0 + RW - 1;
    const int s1 = last_q / kStepKeys + 1;
    j_active_end = nst0 + (s1 < nst1 ? s1 : nst1);
  }

  // ---- HBM -> LDS.  Load i of a wave covers LDS bytes [(wave*LPW+i)*1024, +1024) of a tensor:
  //      row r = (wave*LPW+i)*rowsPerInstr + lane/chunks, chunk slot lane%chunks, which receives
  //      global chunk (slot ^ swizzle(r)).  For a full step the lane's byte offset from the
  //      step's first row is a per-span constant (off_k / off_v).
  int ld_row[LPW];
  unsigned ld_ck[LPW], ld_cv[LPW];  // byte offset of the global chunk inside its row (K / V swizzle)
#pragma unroll
  for (int i = 0; i < LPW; ++i) {
    const int r = (wave * LPW + i) * G::kRowsPerInstr + lane / G::kChunks;
    const int slot_chunk = lane % G::kChunks;
    ld_row[i] = r;
    ld_ck[i] = (unsigned)((slot_chunk ^ G::swz_k(r)) * 16);
    ld_cv[i] = (unsigned)((slot_chunk ^ G::swz_v(r)) * 16);
  }
  unsigned off_k[LPW], off_v[LPW];
  int off_span = -1;
  LDS_AS unsigned char *const lds = (LDS_AS unsigned char *)smem;

  auto issue = [&](int js) {  // enqueue the loads of step js (js < n) into its ring slot
    const int s1 = js >= nst0 ? 1 : 0;
    const int j0 = (s1 ? js - nst0 : js) * kStepKeys;
    const int nrows = s1 ? w.n1 : w.n0;
    const unsigned stride_b = (unsigned)((s1 ? w.stride1 : w.stride0) * 2);
    const unsigned char *kp = (const unsigned char *)(s1 ? w.k1 : w.k0) + (long long)j0 * stride_b;
    const unsigned char *vp = (const unsigned char *)(s1 ? w.v1 : w.v0) + (long long)j0 * stride_b;
    const int nvalid = nrows - j0;  // >= 1; rows past it are clamped (and masked by the consumer)
    LDS_AS unsigned char *dst = lds + (js % kSlots) * G::kSlotBytes + wave * LPW * 1024;
    if (off_span != s1) {
      off_span = s1;
#pragma unroll
      for (int i = 0; i < LPW; ++i) {
        off_k[i] = (unsigned)ld_row[i] * stride_b + ld_ck[i];
        off_v[i] = (unsigned)ld_row[i] * stride_b + ld_cv[i];
      }
    }
    if (nvalid >= kStepKeys) {
#pragma unroll
      for (int i = 0; i < LPW; ++i) {
        __builtin_amdgcn_global_load_lds((const GLB_AS void *)(kp + off_k[i]), (LDS_AS void *)(dst + i * 1024), 16, 0, 0);
        __builtin_amdgcn_global_load_lds((const GLB_AS void *)(vp + off_v[i]),
                                         (LDS_AS void *)(dst + G::kTensorBytes + i * 1024), 16, 0, 0);
      }
    } else {
#pragma unroll
      for (int i = 0; i < LPW; ++i) {
        const int r = ld_row[i] < nvalid ? ld_row[i] : nvalid - 1;
        const unsigned ro = (unsigned)r * stride_b;
        __builtin_amdgcn_global_load_lds((const GLB_AS void *)(kp + (ro + ld_ck[i])), (LDS_AS void *)(dst + i * 1024),
                                         16, 0, 0);
        __builtin_amdgcn_global_load_lds((const GLB_AS void *)(vp + (ro + ld_cv[i])),
                                         (LDS_AS void *)(dst + G::kTensorBytes + i * 1024), 16, 0, 0);
      }
    }
  };
  // Before computing step j: the loads of steps <= j+1 have landed for every wave; then the
  // loads of step j+3 are enqueued (their slot was last read in step j-1).
  auto sync = [&](int j) {
    if (j + 2 < n) __builtin_amdgcn_s_waitcnt(0x0F70 | (2 * LPW));  // vmcnt(2*LPW): step j+2 may be in flight
    else __builtin_amdgcn_s_waitcnt(0x0F70);                        // vmcnt(0)
    __builtin_amdgcn_s_barrier();
    if (j + 3 < n) issue(j + 3);
  };

  issue(0);
  if (1 < n) issue(1);
  if (2 < n) issue(2);

  // ---- Q^T operands: Qr[qb][kc] = Q[row(qb, col)][16 kc + 8 hi .. +7]
  bf16x8 Qr[QB][NC];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    int t = tw0 + 32 * qb + col;
    t = t < last_row ? t : last_row;
    const unsigned short *qrow = w.q + ((long long)t * p.Hq + head) * D + 8 * hi;
#pragma unroll
    for (int kc = 0; kc < NC; ++kc) Qr[qb][kc] = __builtin_bit_cast(bf16x8, *(const uint4 *)(qrow + 16 * kc));
  }

  // ---- per-lane LDS read offsets inside a slot
  int koff[NC];  // K operand: row col, chunk 2kc+hi
#pragma unroll
  for (int kc = 0; kc < NC; ++kc) koff[kc] = col * G::kRowBytes + (((2 * kc + hi) ^ G::swz_k(col)) << 4);
  int voff[NB];  // V^T operand: row 4hi + i16/4 (+16 h2 + 8 u), columns 32 nb + 16 g16 + 4 (i16%4) ..+3
  {
    const int vrow = 4 * hi + (i16 >> 2);
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      const int chunk = 4 * nb + 2 * g16 + ((i16 & 3) >> 1);
      voff[nb] = G::kTensorBytes + vrow * G::kRowBytes + ((chunk ^ G::swz_v(vrow)) << 4) + 8 * (i16 & 1);
    }
  }

  f32x16 O[QB][NB];
  float m_ref[QB], l_run[QB];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    m_ref[qb] = -INFINITY;
    l_run[qb] = 0.f;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
      for (int r = 0; r < 16; ++r) O[qb][nb][r] = 0.f;
  }

  // S^T of the step held in ring slot `slot`
  auto compute_s = [&](int slot, f32x16(&S)[QB]) {
    const LDS_AS unsigned char *kb = lds + slot * G::kSlotBytes;
    const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kc = 0; kc < NC; ++kc) {
      const bf16x8 ka = __builtin_bit_cast(bf16x8, *(const LDS_AS uint4 *)(kb + koff[kc]));
#pragma unroll
      for (int qb = 0; qb < QB; ++qb)
        S[qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, Qr[qb][kc], kc == 0 ? zero : S[qb], 0, 0, 0);
    }
  };
  // O^T += V^T . P^T for the step in `slot`.  k-slot e of half-wave hi in chunk h2 is key
  // 16 h2 + 8 (e/4) + 4 hi + e%4 (the accumulator layout of S^T), so V^T is fetched for exactly
  // those keys: two transposing reads of 4 keys each.  The reads are issued by pv_load (inline
  // asm: the compiler would otherwise order the transposing read after every outstanding
  // global->LDS load) and awaited by pv_wait right before the products that consume them.
  auto pv_load = [&](int slot, s16x4(&Vr)[2][NB][2]) {
    const unsigned vb = (unsigned)(size_t)(lds + slot * G::kSlotBytes);
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      const unsigned va = vb + (unsigned)voff[nb];
#pragma unroll
      for (int h2 = 0; h2 < 2; ++h2) {
        asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(Vr[h2][nb][0]) : "v"(va), "n"(16 * h2 * G::kRowBytes));
        asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2"
                     : "=v"(Vr[h2][nb][1])
                     : "v"(va), "n"((16 * h2 + 8) * G::kRowBytes));
      }
    }
  };
  auto pv_wait = [&](s16x4(&Vr)[2][NB][2]) {
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
  auto pv_mma = [&](const s16x4(&Vr)[2][NB][2], const bf16x8(&P)[QB][2]) {
#pragma unroll
    for (int h2 = 0; h2 < 2; ++h2)
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) {
        const bf16x8 va =
            __builtin_bit_cast(bf16x8, __builtin_shufflevector(Vr[h2][nb][0], Vr[h2][nb][1], 0, 1, 2, 3, 4, 5, 6, 7));
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
          O[qb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, P[qb][h2], O[qb][nb], 0, 0, 0);
      }
  };
  auto pv = [&](int slot, const bf16x8(&P)[QB][2]) {
    s16x4 Vr[2][NB][2];
    pv_load(slot, Vr);
    pv_wait(Vr);
    pv_mma(Vr, P);
  };
  // P = exp2(S c - m_ref c) as bf16, its row sums (of the rounded values) and the row maxima of S
  auto softmax = [&](const f32x16(&S)[QB], bf16x8(&P)[QB][2], float(&psum)[QB], float(&rmax)[QB]) {
    const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      const float mc = m_ref[qb] * c;
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
      float mx = fmaxf(S[qb][0], S[qb][1]);
#pragma unroll
      for (int r = 2; r < 16; r += 2) mx = fmaxf(fmaxf(mx, S[qb][r]), S[qb][r + 1]);
      rmax[qb] = mx;
    }
  };
  // Validate the P just formed against the step's own maximum; rescale and redo if needed.
  auto settle = [&](const f32x16(&S)[QB], bf16x8(&P)[QB][2], float(&psum)[QB], float(&rmax)[QB]) {
    bool need[QB];
    float mx[QB];
    bool any = false;
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      mx[qb] = half_max(rmax[qb]);
      need[qb] = mx[qb] > m_ref[qb] + tau;
      any |= need[qb];
    }
    if (__builtin_amdgcn_ballot_w64(any) != 0) {
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) {
        const float m_new = need[qb] ? mx[qb] : m_ref[qb];
        const float alpha = need[qb] ? __builtin_amdgcn_exp2f((m_ref[qb] - m_new) * c) : 1.f;
        m_ref[qb] = m_new;
        l_run[qb] *= alpha;
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
          for (int r = 0; r < 16; ++r) O[qb][nb][r] *= alpha;
      }
      softmax(S, P, psum, rmax);
    }
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) l_run[qb] += psum[qb];
  };
  // One pipelined step j: S^T(j+1) -> Sn, PV of step j-1 with Pp, P(j) <- Sc.
  auto fast_step = [&](int j, auto do_s, const f32x16(&Sc)[QB], f32x16(&Sn)[QB], const bf16x8(&Pp)[QB][2],
                       bf16x8(&Pc)[QB][2]) {
    float psum[QB], rmax[QB];
    s16x4 Vr[2][NB][2];
    pv_load((j - 1) % kSlots, Vr);
    if constexpr (decltype(do_s)::value) compute_s((j + 1) % kSlots, Sn);
    pv_wait(Vr);
    pv_mma(Vr, Pp);
    softmax(Sc, Pc, psum, rmax);
    settle(Sc, Pc, psum, rmax);
  };
  // An unpipelined step with element masks: keys with in-span index >= lim[qb] are invisible.
  auto slow_step = [&](int j) {
    const bool s1 = j >= nst0;
    const int j0 = (s1 ? j - nst0 : j) * kStepKeys;
    f32x16 S[QB];
    bf16x8 P[QB][2];
    float psum[QB], rmax[QB];
    compute_s(j % kSlots, S);
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      int t = tw0 + 32 * qb + col;
      t = t < last_row ? t : last_row;
      const int lim = s1 ? t + 1 : w.n0;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int key = j0 + 8 * (r >> 2) + 4 * hi + (r & 3);
        if (key >= lim) S[qb][r] = -INFINITY;
      }
      float mx = S[qb][0];
#pragma unroll
      for (int r = 1; r < 16; ++r) mx = fmaxf(mx, S[qb][r]);
      mx = half_max(mx);
      const bool need = mx > m_ref[qb] + tau;  // true on the very first step (m_ref = -inf, mx finite)
      const float m_new = need ? mx : m_ref[qb];
      const float alpha = need ? __builtin_amdgcn_exp2f((m_ref[qb] - m_new) * c) : 1.f;
      m_ref[qb] = m_new;
      l_run[qb] *= alpha;
#pragma unroll
      for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int r = 0; r < 16; ++r) O[qb][nb][r] *= alpha;
    }
    softmax(S, P, psum, rmax);
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) l_run[qb] += psum[qb];
    pv(j % kSlots, P);
  };

  // =========================== main sequence ===========================
  sync(0);
  f32x16 Sa[QB], Sb[QB];
  bf16x8 Pa[QB][2], Pb[QB][2];
  int j = 0;
  if (f > 0) {
    {  // step 0 without overlap: exact maximum as the first reference
      float psum[QB], rmax[QB];
      compute_s(0, Sa);
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) {
        float mx = Sa[qb][0];
#pragma unroll
        for (int r = 1; r < 16; ++r) mx = fmaxf(mx, Sa[qb][r]);
        m_ref[qb] = half_max(mx);
      }
      softmax(Sa, Pb, psum, rmax);
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) l_run[qb] = psum[qb];
      if (f > 1) compute_s(1 % kSlots, Sa);
    }
    j = 1;
    while (j + 2 < f) {
      sync(j);
      fast_step(j, std::true_type{}, Sa, Sb, Pb, Pa);
      sync(j + 1);
      fast_step(j + 1, std::true_type{}, Sb, Sa, Pa, Pb);
      j += 2;
    }
    if (f - j == 2) {
      sync(j);
      fast_step(j, std::true_type{}, Sa, Sb, Pb, Pa);
      sync(j + 1);
      fast_step(j + 1, std::false_type{}, Sb, Sa, Pa, Pb);
      j += 2;
    } else if (f - j == 1) {
      sync(j);
      fast_step(j, std::false_type{}, Sa, Sb, Pb, Pa);
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) {
        Pb[qb][0] = Pa[qb][0];
        Pb[qb][1] = Pa[qb][1];
      }
      j += 1;
    }
  }
  // here j == f and, if f > 0, P(f-1) waits in Pb
  bool pending = f > 0;
  for (; j < n; ++j) {
    if (j > 0) sync(j);
    if (pending) {
      pv((j - 1) % kSlots, Pb);
      pending = false;
    }
    if (j < j_active_end) slow_step(j);
  }
  if (pending) pv((n - 1) % kSlots, Pb);

  // ---- epilogue: normalise, write O (row t, head, d) and LSE
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const int t = tw0 + 32 * qb + col;
    const float l = half_sum(l_run[qb]);
    if (t > last_row) continue;
    const float inv = 1.f / l;
    if (hi == 0) w.lse[(long long)head * w.lse_head_stride + t] = m_ref[qb] * p.scale + __logf(l);
    const long long orow = ((long long)t * p.Hq + head) * D;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
      for (int rg = 0; rg < 4; ++rg) {
        const int d = 32 * nb + 8 * rg + 4 * hi;
        const f32x4 o = {O[qb][nb][4 * rg + 0] * inv, O[qb][nb][4 * rg + 1] * inv, O[qb][nb][4 * rg + 2] * inv,
                         O[qb][nb][4 * rg + 3] * inv};
        if (p.out_fp32) {
          *(f32x4 *)((float *)w.out + orow + d) = o;
        } else {
          const bf16x4 hq = __builtin_convertvector(o, bf16x4);
          *(uint2 *)((unsigned short *)w.out + orow + d) = __builtin_bit_cast(uint2, hq);
        }
      }
  }
}

// =============================================================================================
// launch
// =============================================================================================
hipError_t launch_prefill_fp32(const Problem &p, const PrefillArgs &a, long long grid, hipStream_t st);

static int heads_per_wg(const Problem &p) { return (p.g % 4 == 0) ? 4 : (p.g % 2 == 0) ? 2 : 1; }

int prefill_rows_per_workgroup(const Problem &p) {
  if (p.fp32_math) return 64;
  return (4 / heads_per_wg(p)) * 64;
}

template <int D, int HS>
static hipError_t launch_mfma(const Problem &p, const PrefillArgs &a, long long grid, hipStream_t st) {
  constexpr int lds = kSlots * StepGeom<D>::kSlotBytes;
  auto kern = prefill_mfma_kernel<D, HS>;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(256), lds, st, p, a);
  return hipGetLastError();
}

hipError_t launch_prefill(const Problem &p, const PrefillArgs &a, hipStream_t st) {
  const bool fp32 = p.fp32_math != 0;
  const int hs = fp32 ? 1 : heads_per_wg(p);
  const long long grid = (long long)p.B * p.Hkv * (p.g / hs) * a.n_seg * a.q_blocks_per_seg;
  if (grid <= 0 || grid > 0x7fffffffLL) return hipErrorInvalidValue;
  if (fp32) return launch_prefill_fp32(p, a, grid, st);
  if (p.D == 128) {
    if (hs == 4) return launch_mfma<128, 4>(p, a, grid, st);
    if (hs == 2) return launch_mfma<128, 2>(p, a, grid, st);
    return launch_mfma<128, 1>(p, a, grid, st);
  }
  if (hs == 4) return launch_mfma<64, 4>(p, a, grid, st);
  if (hs == 2) return launch_mfma<64, 2>(p, a, grid, st);
  return launch_mfma<64, 1>(p, a, grid, st);
}

}  // namespace segattn
