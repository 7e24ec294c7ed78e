// Prefill kernels of libsegattn: segment-level causal attention (Eq. 12 with the per-head
// context of Eq. 13, Appendix C) for gfx950.
//
//   prefill_mfma_kernel   bf16 MFMA QK^T and PV, online softmax in registers, K/V tiles of
//                         the [prefix | segment] key ranges staged through LDS.
//   prefill_fp32_kernel   validation mode: the same work decomposition and key ranges, plain
//                         fp32 FMA arithmetic, fp32 output.
//
// Both kernels see a workgroup's keys as two spans: span 0 = the prefix the head's policy
// grants (carried tail and/or past rows; every row visible to every query of the
// workgroup) and span 1 = the rows of the query's own segment (causal).  Tiles that lie
// wholly outside a wave's visible range are never computed; element masks are applied only
// to the tiles that straddle the diagonal or the ragged end of a span.
#include "segattn_internal.h"

namespace segattn {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
#define LDS_AS __attribute__((address_space(3)))

constexpr int kTileKeys = 64;

// One workgroup's share of the problem.
struct WorkItem {
  const unsigned short *k0, *v0, *k1, *v1;  // first row of span 0 / span 1 for this KV head
  long long stride0, stride1;               // elements between consecutive rows
  int n0, n1;                               // rows in span 0; rows of the segment present
  const unsigned short *q;                  // row 0 of the segment's queries, head 0
  unsigned char *out;                       // row 0 of the segment's outputs, head 0
  float *lse;                               // lse of (b, head 0, segment row 0)
  long long lse_head_stride;                // floats between heads in lse
  int t0;                                   // first in-segment query row of the workgroup
  int kv, hsub, b;
  bool valid;
};

// blockIdx -> (sequence, KV head, head sub-group, segment, query block), longest work first:
// all PAST workgroups by descending absolute query block, then the others by descending
// in-segment query block.
__device__ inline WorkItem resolve(const Problem &p, const PrefillArgs &a, int bid, int rows_per_wg,
                                   int heads_per_wg) {
  WorkItem w;
  const int nhs = p.g / heads_per_wg;
  const int nqb = a.q_blocks_per_seg;
  const int n_other = p.Hkv - p.n_past;
  const long long past_items = (long long)p.B * p.n_past * nhs * a.n_seg * nqb;
  int seg, qblk, hidx, b, hs;
  if (bid < past_items) {
    const int per = p.B * p.n_past * nhs;
    const int gq = a.n_seg * nqb - 1 - bid / per;
    int rest = bid % per;
    seg = gq / nqb;
    qblk = gq % nqb;
    hs = rest % nhs;
    rest /= nhs;
    hidx = rest % p.n_past;
    b = rest / p.n_past;
  } else {
    const int y = bid - (int)past_items;
    const int per = p.B * n_other * nhs * a.n_seg;
    qblk = nqb - 1 - y / per;
    int rest = y % per;
    hs = rest % nhs;
    rest /= nhs;
    hidx = p.n_past + rest % n_other;
    rest /= n_other;
    b = rest % p.B;
    seg = rest / p.B;
  }
  const int kv = p.order[hidx];
  const int pol = p.policy[kv];
  w.kv = kv;
  w.hsub = hs;
  w.b = b;
  w.t0 = qblk * rows_per_wg;
  const long long kv_stride = (long long)p.Hkv * p.D;
  if (a.cache == nullptr) {  // SEQ mode: prefix read from k/v by absolute position
    const long long N = a.n_rows;
    const long long s = (long long)seg * p.S;
    const long long m_i = (N - s < p.S) ? (N - s) : p.S;
    long long lo = s;
    if (pol & SEGATTN_PAST) lo = 0;
    else if (pol & SEGATTN_TAIL) lo = (s - p.T > 0) ? s - p.T : 0;
    w.n0 = (int)(s - lo);
    w.n1 = (int)m_i;
    w.k0 = a.k + ((long long)b * N + lo) * kv_stride + (long long)kv * p.D;
    w.v0 = a.v + ((long long)b * N + lo) * kv_stride + (long long)kv * p.D;
    w.k1 = a.k + ((long long)b * N + s) * kv_stride + (long long)kv * p.D;
    w.v1 = a.v + ((long long)b * N + s) * kv_stride + (long long)kv * p.D;
    w.stride0 = w.stride1 = kv_stride;
    w.q = a.q + ((long long)b * N + s) * p.Hq * p.D;
    const long long osz = p.out_fp32 ? 4 : 2;
    w.out = (unsigned char *)a.out + ((long long)b * N + s) * p.Hq * p.D * osz;
    w.lse = a.lse + (long long)b * p.Hq * N + s;
    w.lse_head_stride = N;
  } else {  // CTX mode: prefix (and the committed part of the open segment) from the cache
    const int *meta = (const int *)(a.cache + a.geom.meta_off) + ((long long)b * p.Hkv + kv) * kMetaInts;
    int lo, seg_row0;
    window_of(p, kv, meta, lo, seg_row0);
    const int hi = seg_row0 + meta[META_FILL];
    const long long m = a.n_rows;
    w.n0 = hi - lo;
    w.n1 = (int)m;
    w.k0 = (const unsigned short *)(a.cache + k_block_off(p, a.geom, b, kv)) + (long long)lo * p.D;
    w.v0 = (const unsigned short *)(a.cache + v_block_off(p, a.geom, b, kv)) + (long long)lo * p.D;
    w.stride0 = p.D;
    w.k1 = a.k + (long long)b * m * kv_stride + (long long)kv * p.D;
    w.v1 = a.v + (long long)b * m * kv_stride + (long long)kv * p.D;
    w.stride1 = kv_stride;
    w.q = a.q + (long long)b * m * p.Hq * p.D;
    const long long osz = p.out_fp32 ? 4 : 2;
    w.out = (unsigned char *)a.out + (long long)b * m * p.Hq * p.D * osz;
    w.lse = a.lse + (long long)b * p.Hq * m;
    w.lse_head_stride = m;
  }
  w.valid = w.t0 < w.n1;
  return w;
}

__device__ inline float bf16_bits_to_f32(unsigned short h) { return __uint_as_float((unsigned)h << 16); }

// =============================================================================================
// bf16 MFMA kernel
// =============================================================================================
// Workgroup = 4 waves.  HS query heads of one GQA group share the staged K/V tiles; each wave
// owns one head and RW = 32*QB consecutive query rows.  Per wave and 64-key tile:
//   S^T[key][query] = K_tile . Q^T        v_mfma_f32_32x32x16_bf16, A = K rows from LDS
//   online softmax over keys               (a query lives in lane%32 and lane%32+32)
//   O^T[d][query]  += V_tile^T . P^T       A = V^T via ds_read_b64_tr_b16, B = P straight
//                                          from the S^T accumulator registers
// Computing the transposed products makes the accumulator layout of S^T (lane = query, the
// lane's registers = keys) exactly the B-operand layout the PV product wants, so P never
// leaves the register file.
template <int D>
struct TileGeom {
  static constexpr int kStrideK = D * 2 + 16;  // bytes per K row in LDS: 16-lane b128 reads hit 64 banks
  static constexpr int kStrideV = D * 2 + 64;  // bytes per V row: 4 consecutive rows x 64 B hit 64 banks
  static constexpr int kBytesK = kTileKeys * kStrideK;
  static constexpr int kBytesV = kTileKeys * kStrideV;
  static constexpr int kStage = kBytesK + kBytesV;
  static constexpr int kChunksPerRow = D / 8;               // 16-byte chunks
  static constexpr int kPasses = kTileKeys * kChunksPerRow / 256;
  static constexpr int kRowsPerPass = 256 / kChunksPerRow;
};

template <int D, int QB, int HS, int OCC>
__global__ __launch_bounds__(256, OCC) void prefill_mfma_kernel(const Problem p, const PrefillArgs a) {
  using G = TileGeom<D>;
  constexpr int PB = 4 / HS;        // position blocks per workgroup
  constexpr int RW = 32 * QB;       // query rows per wave
  constexpr int BQ = PB * RW;       // query rows per workgroup
  constexpr int NC = D / 16;        // k-chunks of QK^T
  constexpr int NB = D / 32;        // 32-row blocks of O^T
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

  const WorkItem w = resolve(p, a, blockIdx.x, BQ, HS);
  if (!w.valid) return;

  const int tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63;
  const int hi = lane >> 5, col = lane & 31;
  const int head = w.kv * p.g + w.hsub * HS + (wave % HS);
  const int tw0 = w.t0 + (wave / HS) * RW;   // first query row of this wave
  const int last_row = w.n1 - 1;
  const float c = p.scale_log2e;

  // ---- Q^T operands: Qr[qb][kc] = Q[row(qb, col)][16 kc + 8 hi .. +7]
  bf16x8 Qr[QB][NC];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    int t = tw0 + 32 * qb + col;
    t = t < last_row ? t : last_row;
    const unsigned short *qrow = w.q + ((long long)t * p.Hq + head) * D + 8 * hi;
#pragma unroll
    for (int kc = 0; kc < NC; ++kc)
      Qr[qb][kc] = __builtin_bit_cast(bf16x8, *(const uint4 *)(qrow + 16 * kc));
  }

  f32x16 O[QB][NB];
  float m_run[QB], l_run[QB];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    m_run[qb] = -INFINITY;
    l_run[qb] = 0.f;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
      for (int r = 0; r < 16; ++r) O[qb][nb][r] = 0.f;
  }

  // ---- tile schedule: span 0 (prefix), then span 1 up to the workgroup's last query
  const int n1_needed = (w.t0 + BQ < w.n1) ? (w.t0 + BQ) : w.n1;
  const int nt0 = (w.n0 + kTileKeys - 1) / kTileKeys;
  const int nt1 = (n1_needed + kTileKeys - 1) / kTileKeys;
  const int nt = nt0 + nt1;

  const int ld_chunk = tid % G::kChunksPerRow;
  const int ld_row = tid / G::kChunksPerRow;
  uint4 kreg[G::kPasses], vreg[G::kPasses];

  auto issue_loads = [&](int i) {
    const bool s1 = i >= nt0;
    const int j0 = (s1 ? i - nt0 : i) * kTileKeys;
    const int nrows = s1 ? w.n1 : w.n0;
    const unsigned short *kp = s1 ? w.k1 : w.k0;
    const unsigned short *vp = s1 ? w.v1 : w.v0;
    const long long stride = s1 ? w.stride1 : w.stride0;
#pragma unroll
    for (int ps = 0; ps < G::kPasses; ++ps) {
      int row = j0 + ld_row + ps * G::kRowsPerPass;
      row = row < nrows ? row : nrows - 1;
      const long long off = (long long)row * stride + ld_chunk * 8;
      kreg[ps] = *(const uint4 *)(kp + off);
      vreg[ps] = *(const uint4 *)(vp + off);
    }
  };
  auto store_lds = [&](int stage) {
    unsigned char *ks = smem + stage * G::kStage;
    unsigned char *vs = ks + G::kBytesK;
#pragma unroll
    for (int ps = 0; ps < G::kPasses; ++ps) {
      const int row = ld_row + ps * G::kRowsPerPass;
      *(uint4 *)(ks + row * G::kStrideK + ld_chunk * 16) = kreg[ps];
      *(uint4 *)(vs + row * G::kStrideV + ld_chunk * 16) = vreg[ps];
    }
  };

  issue_loads(0);
  store_lds(0);
  __syncthreads();

  for (int i = 0; i < nt; ++i) {
    if (i + 1 < nt) issue_loads(i + 1);

    const bool s1 = i >= nt0;
    const int j0 = (s1 ? i - nt0 : i) * kTileKeys;
    // span 1: a wave has nothing to do in tiles that start after its last query
    const bool active = !s1 || j0 <= tw0 + RW - 1;
    if (active) {
      const unsigned char *ks = smem + (i & 1) * G::kStage;
      const unsigned char *vs = ks + G::kBytesK;

      // ---- S^T = K . Q^T  (two 32-key blocks x QB query blocks)
      f32x16 S[2][QB];
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
#pragma unroll
          for (int r = 0; r < 16; ++r) S[kb][qb][r] = 0.f;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) {
        const unsigned char *krow = ks + (32 * kb + col) * G::kStrideK + 16 * hi;
#pragma unroll
        for (int kc = 0; kc < NC; ++kc) {
          const bf16x8 ka = __builtin_bit_cast(bf16x8, *(const uint4 *)(krow + 32 * kc));
#pragma unroll
          for (int qb = 0; qb < QB; ++qb)
            S[kb][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, Qr[qb][kc], S[kb][qb], 0, 0, 0);
        }
      }

      // ---- masks: only on tiles that touch the end of span 0 or the diagonal of span 1
      const int nrows = s1 ? w.n1 : w.n0;
      const bool need_mask = s1 ? (j0 + kTileKeys - 1 > tw0) : (j0 + kTileKeys > nrows);
      if (need_mask) {
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
          int t = tw0 + 32 * qb + col;
          t = t < last_row ? t : last_row;
          const int lim = s1 ? t + 1 : nrows;  // keys with index < lim are visible
#pragma unroll
          for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
              const int key = j0 + 32 * kb + 8 * (r >> 2) + 4 * hi + (r & 3);
              if (key >= lim) S[kb][qb][r] = -INFINITY;
            }
        }
      }

      // ---- online softmax (per query: lanes col and col+32 hold its 2x32 keys of the tile)
      bf16x8 P[2][QB][2];
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) {
        float mx = m_run[qb];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int r = 0; r < 16; ++r) mx = fmaxf(mx, S[kb][qb][r]);
        {
          const int mi = __float_as_int(mx);
          const auto sw = __builtin_amdgcn_permlane32_swap(mi, mi, false, false);
          mx = fmaxf(__int_as_float(sw[0]), __int_as_float(sw[1]));
        }
        const float alpha = __builtin_amdgcn_exp2f((m_run[qb] - mx) * c);
        const float mc = mx * c;
        float psum = 0.f;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
          float pv[16];
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            pv[r] = __builtin_amdgcn_exp2f(fmaf(S[kb][qb][r], c, -mc));
            psum += pv[r];
          }
#pragma unroll
          for (int h2 = 0; h2 < 2; ++h2) {
            f32x8 f;
#pragma unroll
            for (int e = 0; e < 8; ++e) f[e] = pv[8 * h2 + e];
            P[kb][qb][h2] = __builtin_convertvector(f, bf16x8);
          }
        }
        l_run[qb] = l_run[qb] * alpha + psum;
        m_run[qb] = mx;
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
          for (int r = 0; r < 16; ++r) O[qb][nb][r] *= alpha;
      }

      // ---- O^T += V^T . P^T.  k-slot e of half-wave hi in chunk (kb, h2) is key
      //      32 kb + 16 h2 + 8 (e/4) + 4 hi + e%4 (the accumulator layout of S^T), so V^T is
      //      fetched for exactly those keys: two transposing LDS reads of 4 keys each.
      const int i16 = lane & 15, g16 = (lane >> 4) & 1;
      const LDS_AS unsigned char *vbase =
          (const LDS_AS unsigned char *)vs + (4 * hi + (i16 >> 2)) * G::kStrideV + (16 * g16 + 4 * (i16 & 3)) * 2;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int h2 = 0; h2 < 2; ++h2) {
          const LDS_AS unsigned char *vk = vbase + (32 * kb + 16 * h2) * G::kStrideV;
#pragma unroll
          for (int nb = 0; nb < NB; ++nb) {
            const s16x4 lo4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4 *)(vk + nb * 64));
            const s16x4 hi4 =
                __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4 *)(vk + 8 * G::kStrideV + nb * 64));
            const s16x8 va = __builtin_shufflevector(lo4, hi4, 0, 1, 2, 3, 4, 5, 6, 7);
            const bf16x8 vb = __builtin_bit_cast(bf16x8, va);
#pragma unroll
            for (int qb = 0; qb < QB; ++qb)
              O[qb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vb, P[kb][qb][h2], O[qb][nb], 0, 0, 0);
          }
        }
    }

    if (i + 1 < nt) store_lds((i + 1) & 1);
    __syncthreads();
  }

  // ---- epilogue: normalise, write O (row t, head, d) and LSE
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const int t = tw0 + 32 * qb + col;
    float l = l_run[qb];
    {
      const int li = __float_as_int(l);
      const auto sw = __builtin_amdgcn_permlane32_swap(li, li, false, false);
      l = __int_as_float(sw[0]) + __int_as_float(sw[1]);
    }
    if (t > last_row) continue;
    const float inv = 1.f / l;
    if (hi == 0) w.lse[(long long)head * w.lse_head_stride + t] = m_run[qb] * p.scale + __logf(l);
    const long long orow = ((long long)t * p.Hq + head) * D;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
      for (int rg = 0; rg < 4; ++rg) {
        const int d = 32 * nb + 8 * rg + 4 * hi;
        const float o0 = O[qb][nb][4 * rg + 0] * inv, o1 = O[qb][nb][4 * rg + 1] * inv;
        const float o2 = O[qb][nb][4 * rg + 2] * inv, o3 = O[qb][nb][4 * rg + 3] * inv;
        if (p.out_fp32) {
          *(float4 *)((float *)w.out + orow + d) = make_float4(o0, o1, o2, o3);
        } else {
          typedef float f32x4 __attribute__((ext_vector_type(4)));
          typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
          const f32x4 f = {o0, o1, o2, o3};
          const bf16x4 hq = __builtin_convertvector(f, bf16x4);
          *(uint2 *)((unsigned short *)w.out + orow + d) = __builtin_bit_cast(uint2, hq);
        }
      }
  }
}

// =============================================================================================
// fp32 validation kernel
// =============================================================================================
// 64 query rows of one head per workgroup; thread (row, part) handles the keys j = part mod 4
// of each 32-key tile with scalar fp32 FMAs and merges the four partial softmax states with
// wave shuffles at the end.
template <int D>
__global__ __launch_bounds__(256) void prefill_fp32_kernel(const Problem p, const PrefillArgs a) {
  constexpr int BQ = 64, TK = 32, LD = D + 4;
  __shared__ __attribute__((aligned(16))) float Ks[TK * LD];
  __shared__ __attribute__((aligned(16))) float Vs[TK * LD];
  const WorkItem w = resolve(p, a, blockIdx.x, BQ, 1);
  if (!w.valid) return;
  const int tid = threadIdx.x;
  const int r = tid >> 2, part = tid & 3;
  const int head = w.kv * p.g + w.hsub;
  const int t_raw = w.t0 + r;
  const int t = t_raw < w.n1 ? t_raw : w.n1 - 1;

  float qv[D], acc[D];
  {
    const unsigned short *qrow = w.q + ((long long)t * p.Hq + head) * D;
#pragma unroll
    for (int d = 0; d < D; ++d) {
      qv[d] = bf16_bits_to_f32(qrow[d]);
      acc[d] = 0.f;
    }
  }
  float m_run = -INFINITY, l_run = 0.f;
  const int n1_needed = (w.t0 + BQ < w.n1) ? (w.t0 + BQ) : w.n1;

  for (int span = 0; span < 2; ++span) {
    const int nrows = span ? w.n1 : w.n0;
    const int nvis = span ? n1_needed : w.n0;
    const unsigned short *kp = span ? w.k1 : w.k0;
    const unsigned short *vp = span ? w.v1 : w.v0;
    const long long stride = span ? w.stride1 : w.stride0;
    for (int j0 = 0; j0 < nvis; j0 += TK) {
      __syncthreads();
      for (int e = tid; e < TK * D; e += 256) {
        const int jr = e / D, d = e % D;
        int row = j0 + jr;
        row = row < nrows ? row : nrows - 1;
        Ks[jr * LD + d] = bf16_bits_to_f32(kp[(long long)row * stride + d]);
        Vs[jr * LD + d] = bf16_bits_to_f32(vp[(long long)row * stride + d]);
      }
      __syncthreads();
      const int lim = span ? t + 1 : nrows;
      float sc[TK / 4];
      float tmax = -INFINITY;
#pragma unroll
      for (int jj = 0; jj < TK / 4; ++jj) {
        const int jr = part + 4 * jj;
        float s = 0.f;
#pragma unroll
        for (int d = 0; d < D; d += 4) {
          const float4 kk = *(const float4 *)&Ks[jr * LD + d];
          s = fmaf(qv[d], kk.x, s);
          s = fmaf(qv[d + 1], kk.y, s);
          s = fmaf(qv[d + 2], kk.z, s);
          s = fmaf(qv[d + 3], kk.w, s);
        }
        s *= p.scale;
        sc[jj] = (j0 + jr < lim) ? s : -INFINITY;
        tmax = fmaxf(tmax, sc[jj]);
      }
      if (tmax == -INFINITY) continue;  // nothing visible for this thread in this tile
      const float m_new = fmaxf(m_run, tmax);
      const float alpha = expf(m_run - m_new);  // exp(-inf) = 0 on the first visible tile
      l_run *= alpha;
#pragma unroll
      for (int d = 0; d < D; ++d) acc[d] *= alpha;
#pragma unroll
      for (int jj = 0; jj < TK / 4; ++jj) {
        if (sc[jj] == -INFINITY) continue;
        const int jr = part + 4 * jj;
        const float pr = expf(sc[jj] - m_new);
        l_run += pr;
#pragma unroll
        for (int d = 0; d < D; d += 4) {
          const float4 vv = *(const float4 *)&Vs[jr * LD + d];
          acc[d] = fmaf(pr, vv.x, acc[d]);
          acc[d + 1] = fmaf(pr, vv.y, acc[d + 1]);
          acc[d + 2] = fmaf(pr, vv.z, acc[d + 2]);
          acc[d + 3] = fmaf(pr, vv.w, acc[d + 3]);
        }
      }
      m_run = m_new;
    }
  }
  // merge the four parts of a row (adjacent lanes)
#pragma unroll
  for (int sh = 1; sh <= 2; sh <<= 1) {
    const float m_o = __shfl_xor(m_run, sh);
    const float l_o = __shfl_xor(l_run, sh);
    const float m_new = fmaxf(m_run, m_o);
    const float a_s = (m_run == -INFINITY) ? 0.f : expf(m_run - m_new);
    const float a_o = (m_o == -INFINITY) ? 0.f : expf(m_o - m_new);
    l_run = l_run * a_s + l_o * a_o;
#pragma unroll
    for (int d = 0; d < D; ++d) {
      const float o = __shfl_xor(acc[d], sh);
      acc[d] = acc[d] * a_s + o * a_o;
    }
    m_run = m_new;
  }
  if (t_raw >= w.n1) return;
  if (part == 0) w.lse[(long long)head * w.lse_head_stride + t] = m_run + logf(l_run);
  const float inv = 1.f / l_run;
  float *orow = (float *)w.out + ((long long)t * p.Hq + head) * D;
  for (int d = part * (D / 4); d < (part + 1) * (D / 4); ++d) orow[d] = acc[d] * inv;
}

// =============================================================================================
// launch
// =============================================================================================
static int heads_per_wg(const Problem &p) { return (p.g % 4 == 0) ? 4 : (p.g % 2 == 0) ? 2 : 1; }

int prefill_rows_per_workgroup(const Problem &p) {
  if (p.fp32_math) return 64;
  return (4 / heads_per_wg(p)) * 64;
}

template <int D, int QB, int HS, int OCC>
static hipError_t launch_mfma(const Problem &p, const PrefillArgs &a, long long grid, hipStream_t st) {
  constexpr int lds = 2 * TileGeom<D>::kStage;
  auto kern = prefill_mfma_kernel<D, QB, HS, OCC>;
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
  if (fp32) {
    if (p.D == 128) hipLaunchKernelGGL(prefill_fp32_kernel<128>, dim3((unsigned)grid), dim3(256), 0, st, p, a);
    else hipLaunchKernelGGL(prefill_fp32_kernel<64>, dim3((unsigned)grid), dim3(256), 0, st, p, a);
    return hipGetLastError();
  }
  if (p.D == 128) {
    if (hs == 4) return launch_mfma<128, 2, 4, 1>(p, a, grid, st);
    if (hs == 2) return launch_mfma<128, 2, 2, 1>(p, a, grid, st);
    return launch_mfma<128, 2, 1, 1>(p, a, grid, st);
  }
  if (hs == 4) return launch_mfma<64, 2, 4, 1>(p, a, grid, st);
  if (hs == 2) return launch_mfma<64, 2, 2, 1>(p, a, grid, st);
  return launch_mfma<64, 2, 1, 1>(p, a, grid, st);
}

}  // namespace segattn
