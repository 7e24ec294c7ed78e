// Decode path of libsegattn: one new token per sequence attends over the visible window
// [prefix | open segment] of every KV head (Eq. 12 / Eq. 13 for a single query row; Eq. 2's
// conditioning on x_<t, C_{i-1}, R_{i-1}).  The work is HBM-bound (every visible K and V row
// is read once per KV head and serves the g query heads of the group), so it is a split-K
// reduction over an even partition of the rows:
//   split kernel           the windows of all (sequence, KV head) pairs are laid end to end and cut
//                          into one slice of rows_per_wg rows per workgroup, as many workgroups as
//                          the chip holds at once; at the end of every window a workgroup touches
//                          it writes one partial (acc[D], m, l) per query head.
//   decode_combine_kernel  one workgroup per (b, query head): merges the partials of its window.
// Equal slices instead of fixed chunks: no empty workgroups, no uneven tail, and few partials --
// the partials' stores, spread over tens of MB in the middle of the read stream, cost a fixed-chunk
// version 13 % of its time.
// Two split kernels.  The bf16 path runs on the matrix cores (segattn_decode_mfma.hip).  The one
// in this file works on the vector ALUs: a workgroup streams its slice with 16-byte coalesced
// loads (D/8 lanes per key row), forms the dot products per row with v_dot2 and a DPP reduction
// inside each lane group, keeps an online-softmax state per lane group and merges the groups with
// wave shuffles and the four waves through LDS.  It is the fp32 validation form (EXACT: fp32 FMAs,
// unrounded weights); its bf16 instantiations (SEGATTN_DECODE_MFMA_MIN_G above the group size
// selects them) reach the same speed for groups of up to four heads and are bound by their ~150
// instructions per row and lane group beyond that.
#include "segattn_decode_slices.h"

#ifndef SEGATTN_DECODE_MFMA_MIN_G
#define SEGATTN_DECODE_MFMA_MIN_G 1
#endif
#ifndef SEGATTN_DECODE_WAVES
#define SEGATTN_DECODE_WAVES 3
#endif
#ifndef SEGATTN_DECODE_U
#define SEGATTN_DECODE_U 8
#endif

namespace segattn {

// sum over the LPR lanes of a lane group (LPR = 8 or 16), result in every lane of the group
template <int LPR>
__device__ inline float group_sum(float x) {
  x += __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(x), 0xB1, 0xF, 0xF, true));   // quad_perm [1,0,3,2]
  x += __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(x), 0x4E, 0xF, 0xF, true));   // quad_perm [2,3,0,1]
  x += __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(x), 0x141, 0xF, 0xF, true));  // row_half_mirror
  if (LPR == 16) x += __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(x), 0x140, 0xF, 0xF, true));  // row_mirror
  return x;
}

__device__ inline void unpack8(const uint4 u, float (&f)[8]) {
  f[0] = __uint_as_float(u.x << 16); f[1] = __uint_as_float(u.x & 0xffff0000u);
  f[2] = __uint_as_float(u.y << 16); f[3] = __uint_as_float(u.y & 0xffff0000u);
  f[4] = __uint_as_float(u.z << 16); f[5] = __uint_as_float(u.z & 0xffff0000u);
  f[6] = __uint_as_float(u.w << 16); f[7] = __uint_as_float(u.w & 0xffff0000u);
}

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

// 16-byte load of data that is read once: marked non-temporal so that the 2-3 GB of K/V rows a
// decode step streams do not displace each other in the caches on their way (measured +7 %).
__device__ inline uint4 load_stream(const uint4 *ptr) {
  const u32x4 x = __builtin_nontemporal_load((const u32x4 *)ptr);
  return make_uint4(x.x, x.y, x.z, x.w);
}

__device__ inline float dot2_bf16(unsigned a, unsigned b, float c) {  // a.lo*b.lo + a.hi*b.hi + c
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, a), __builtin_bit_cast(bf16x2, b), c, false);
}

// EXACT: fp32 weights and fp32 FMAs throughout (validation mode).  Otherwise the dot products
// use v_dot2_f32_bf16 on the bf16 pairs as they come from memory, and the weights are rounded to
// bf16 for the PV product (as in the prefill kernel; the row sums use the same rounded values).
template <int D, int GH, bool EXACT>
__global__ __launch_bounds__(256, GH == 8 ? 2 : SEGATTN_DECODE_WAVES) void decode_split_kernel(const Problem p, const DecodeArgs a,
                                                          const int head_pass) {
  constexpr int LPR = D / 8;        // lanes per key row
  constexpr int GPW = 64 / LPR;     // key rows per wave-wide load
  constexpr int U = GH == 8 ? SEGATTN_DECODE_U / 2 : SEGATTN_DECODE_U;  // rows in flight per lane group
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int grp = lane / LPR, li = lane % LPR;
  const float c = p.scale_log2e;

  __shared__ float sm_m[4][GH], sm_l[4][GH];
  __shared__ __align__(16) float sm_acc[4][GH][D];

  // ---- where this workgroup's slice [start, start + rows_per_wg) of the concatenated windows begins
  const int n_win = p.B * p.Hkv;
  const long long start = (long long)blockIdx.x * a.rows_per_wg;
  int w, off;
  decode_slice_start(p, a, start, w, off);
  if (w < 0) return;  // the slices before this one cover every row
  // this workgroup's ordinal among those that touch window w (windows it enters later start in it)
  int split = (int)((long long)blockIdx.x - (start - off) / a.rows_per_wg);
  int remaining = a.rows_per_wg;
  int *counts = ws_counts(a.cache, a.geom);
  float *slots = ws_slots(a.cache, a.geom, p);

  for (; remaining > 0 && w < n_win; ++w, off = 0, split = 0) {
    const int b = w / p.Hkv, kv = w % p.Hkv;
    int lo, hi;
    decode_window_rows(p, a, w, lo, hi);
    lo = __builtin_amdgcn_readfirstlane(lo);
    hi = __builtin_amdgcn_readfirstlane(hi);
    const int c0 = lo + off;
    const int c1 = min(hi, c0 + remaining);
    if (c1 <= c0) continue;
    remaining -= c1 - c0;
    const int head0 = kv * p.g + head_pass * GH;
    // heads of the group this pass covers; with a group size that is no multiple of GH the last
    // pass computes surplus heads on a repeated query row and drops them
    const int live = min(GH, p.g - head_pass * GH);

    uint4 qp[GH];   // this lane's 8 query elements per head, as bf16 pairs
    float qf[EXACT ? GH : 1][8];
#pragma unroll
    for (int h = 0; h < GH; ++h) {
      qp[h] = *(const uint4 *)(a.q + ((long long)b * p.Hq + head0 + (h < live ? h : live - 1)) * D + li * 8);
      if (EXACT) unpack8(qp[h], qf[h]);
    }

    float m_run[GH], l_run[GH], acc[GH][8];
#pragma unroll
    for (int h = 0; h < GH; ++h) {
      m_run[h] = -INFINITY;
      l_run[h] = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[h][e] = 0.f;
    }

    const uint4 *kb = (const uint4 *)(a.cache + attn_k_off(p, a.geom, b, kv)) + li;
    const uint4 *vb = (const uint4 *)(a.cache + attn_v_off(p, a.geom, b, kv)) + li;
    constexpr int ROWS_PER_ITER = 4 * GPW * U;  // rows a workgroup consumes per iteration
    for (int r0 = c0; r0 < c1; r0 += ROWS_PER_ITER) {
      uint4 kr[U], vr[U];
      int row[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        row[u] = r0 + (u * 4 + wave) * GPW + grp;
        const int rc = row[u] < c1 ? row[u] : c1 - 1;   // clamp: stays inside the window
        kr[u] = load_stream(kb + (long long)rc * LPR);
        vr[u] = load_stream(vb + (long long)rc * LPR);
      }
      float s[U][GH];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        float kf[8];
        if (EXACT) unpack8(kr[u], kf);
#pragma unroll
        for (int h = 0; h < GH; ++h) {
          float d = 0.f;
          if (EXACT) {
#pragma unroll
            for (int e = 0; e < 8; ++e) d = fmaf(qf[h][e], kf[e], d);
          } else {
            d = dot2_bf16(qp[h].x, kr[u].x, d);
            d = dot2_bf16(qp[h].y, kr[u].y, d);
            d = dot2_bf16(qp[h].z, kr[u].z, d);
            d = dot2_bf16(qp[h].w, kr[u].w, d);
          }
          d = group_sum<LPR>(d);
          s[u][h] = row[u] < c1 ? d : -INFINITY;
        }
      }
      if (row[0] >= c1) continue;  // whole lane group past the end (rows ascend with u)
      float pw[U][GH];
      unsigned pp[U / 2][GH];  // weights of rows (2i, 2i+1) as a bf16 pair
#pragma unroll
      for (int h = 0; h < GH; ++h) {
        float mx = m_run[h];
#pragma unroll
        for (int u = 0; u < U; ++u) mx = fmaxf(mx, s[u][h]);
        const float alpha = __builtin_amdgcn_exp2f((m_run[h] - mx) * c);
        const float mc = mx * c;
        float ps = 0.f;
#pragma unroll
        for (int u = 0; u < U; ++u) pw[u][h] = __builtin_amdgcn_exp2f(fmaf(s[u][h], c, -mc));
        if (EXACT) {
#pragma unroll
          for (int u = 0; u < U; ++u) ps += pw[u][h];
        } else {
#pragma unroll
          for (int i = 0; i < U / 2; ++i) {
            const f32x2 two = {pw[2 * i][h], pw[2 * i + 1][h]};
            pp[i][h] = __builtin_bit_cast(unsigned, __builtin_convertvector(two, bf16x2));
            ps = dot2_bf16(pp[i][h], 0x3f803f80u, ps);
          }
        }
        l_run[h] = l_run[h] * alpha + ps;
        m_run[h] = mx;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[h][e] *= alpha;
      }
      if (EXACT) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
          float vf[8];
          unpack8(vr[u], vf);
#pragma unroll
          for (int h = 0; h < GH; ++h)
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[h][e] = fmaf(pw[u][h], vf[e], acc[h][e]);
        }
      } else {
#pragma unroll
        for (int i = 0; i < U / 2; ++i) {
          // element e of rows 2i and 2i+1 side by side: low halves then high halves of each word
          const unsigned w0[4] = {vr[2 * i].x, vr[2 * i].y, vr[2 * i].z, vr[2 * i].w};
          const unsigned w1[4] = {vr[2 * i + 1].x, vr[2 * i + 1].y, vr[2 * i + 1].z, vr[2 * i + 1].w};
          unsigned vpair[8];
#pragma unroll
          for (int wd = 0; wd < 4; ++wd) {
            vpair[2 * wd] = __builtin_amdgcn_perm(w1[wd], w0[wd], 0x05040100u);
            vpair[2 * wd + 1] = __builtin_amdgcn_perm(w1[wd], w0[wd], 0x07060302u);
          }
#pragma unroll
          for (int h = 0; h < GH; ++h)
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[h][e] = dot2_bf16(vpair[e], pp[i][h], acc[h][e]);
        }
      }
    }

    // ---- this window's partial: merge the lane groups of a wave (shuffles), then the four waves (LDS)
#pragma unroll
    for (int h = 0; h < GH; ++h) {
#pragma unroll
      for (int sh = LPR; sh < 64; sh <<= 1) {
        const float m_o = __shfl_xor(m_run[h], sh);
        const float l_o = __shfl_xor(l_run[h], sh);
        const float mx = fmaxf(m_run[h], m_o);
        const float a_s = (m_run[h] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f((m_run[h] - mx) * c);
        const float a_o = (m_o == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f((m_o - mx) * c);
        l_run[h] = l_run[h] * a_s + l_o * a_o;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float o = __shfl_xor(acc[h][e], sh);
          acc[h][e] = acc[h][e] * a_s + o * a_o;
        }
        m_run[h] = mx;
      }
    }
    __syncthreads();  // the previous window's partial has been read out of LDS
    if (grp == 0) {
#pragma unroll
      for (int h = 0; h < GH; ++h) {
        if (li == 0) {
          sm_m[wave][h] = m_run[h];
          sm_l[wave][h] = l_run[h];
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) sm_acc[wave][h][li * 8 + e] = acc[h][e];
      }
    }
    __syncthreads();
    for (int idx = tid; idx < GH * D / 4; idx += 256) {  // one float4 of one head's partial per thread
      const int h = idx / (D / 4), d = (idx % (D / 4)) * 4;
      float mx = -INFINITY;
#pragma unroll
      for (int wv = 0; wv < 4; ++wv) mx = fmaxf(mx, sm_m[wv][h]);
      float l = 0.f;
      float4 o = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int wv = 0; wv < 4; ++wv) {
        const float wgt = (sm_m[wv][h] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f((sm_m[wv][h] - mx) * c);
        const float4 x = *(const float4 *)&sm_acc[wv][h][d];
        l += sm_l[wv][h] * wgt;
        o.x += x.x * wgt;
        o.y += x.y * wgt;
        o.z += x.z * wgt;
        o.w += x.w * wgt;
      }
      if (h >= live) continue;
      float *slot = slots + (ws_slot_base(p, a.geom, b, head0 + h) + split) * ws_slot_floats(D);
      *(float4 *)(slot + d) = o;
      if (d == 0) *(float2 *)(slot + D) = float2{mx, l};
    }
    if (tid == 0 && c1 == hi && head_pass == 0) counts[w] = split + 1;  // the window's last rows are here
  }
}

// One workgroup per (b, query head).  All threads find the global maximum over the splits; then
// wave w accumulates the splits congruent to w mod 4 (lanes over the D outputs) and the four
// partial sums meet in LDS.
template <int D>
__global__ __launch_bounds__(256) void decode_combine_kernel(const Problem p, const DecodeArgs a) {
  const int b = blockIdx.x / p.Hq, head = blockIdx.x % p.Hq;
  const int kv = head / p.g;
  const int ns = ws_counts(a.cache, a.geom)[b * p.Hkv + kv];
  const float *ws = ws_slots(a.cache, a.geom, p) + ws_slot_base(p, a.geom, b, head) * ws_slot_floats(D);
  constexpr int SF = D + kWsTailFloats;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const float c = p.scale_log2e;
  constexpr int DPL = D / 64;
  __shared__ float sm_max[4], sm_l[4], sm_o[4][D];

  float mx = -INFINITY;
  for (int s = tid; s < ns; s += 256) mx = fmaxf(mx, ws[(long long)s * SF + D]);
#pragma unroll
  for (int sh = 1; sh < 64; sh <<= 1) mx = fmaxf(mx, __shfl_xor(mx, sh));
  if (lane == 0) sm_max[wave] = mx;
  __syncthreads();
  mx = fmaxf(fmaxf(sm_max[0], sm_max[1]), fmaxf(sm_max[2], sm_max[3]));

  float l = 0.f, o[DPL];
#pragma unroll
  for (int e = 0; e < DPL; ++e) o[e] = 0.f;
#pragma unroll 4
  for (int s = wave; s < ns; s += 4) {
    const float *slot = ws + (long long)s * SF;
    const float wgt = __builtin_amdgcn_exp2f((slot[D] - mx) * c);
    l = fmaf(slot[D + 1], wgt, l);
#pragma unroll
    for (int e = 0; e < DPL; ++e) o[e] = fmaf(slot[lane * DPL + e], wgt, o[e]);
  }
  if (lane == 0) sm_l[wave] = l;
#pragma unroll
  for (int e = 0; e < DPL; ++e) sm_o[wave][lane * DPL + e] = o[e];
  __syncthreads();
  if (tid >= D) return;
  l = (sm_l[0] + sm_l[1]) + (sm_l[2] + sm_l[3]);
  const float od = (sm_o[0][tid] + sm_o[1][tid]) + (sm_o[2][tid] + sm_o[3][tid]);
  const float r = od / l;
  const long long oidx = ((long long)b * p.Hq + head) * D + tid;
  if (p.out_fp32) ((float *)a.out)[oidx] = r;
  else ((__bf16 *)a.out)[oidx] = (__bf16)r;
  if (tid == 0) a.lse[(long long)b * p.Hq + head] = mx * p.scale + __logf(l);
}

// Workgroups of the split kernel the chip holds at once (per instantiation, asked once).
template <int D, int GH, bool EXACT>
static int resident_workgroups() {
  static ResidentCount count;
  return count.get((const void *)decode_split_kernel<D, GH, EXACT>, 256, 0);
}

template <int D, int GH, bool EXACT>
static hipError_t launch_split_gh(const Problem &p, DecodeArgs a, hipStream_t st) {
  const int resident = resident_workgroups<D, GH, EXACT>();
  if (resident == 0) return hipErrorUnknown;
  // equal slices, one per resident workgroup, but never shorter than the chunk the workspace is sized for
  long long per = (a.total_rows + resident - 1) / resident;
  if (per < a.geom.decode_chunk) per = a.geom.decode_chunk;
  per = (per + 127) / 128 * 128;
  if (per > 0x7fffff00LL) return hipErrorInvalidValue;
  a.rows_per_wg = (int)per;
  const long long blocks = (a.total_rows + per - 1) / per;
  for (int pass = 0; pass < (p.g + GH - 1) / GH; ++pass) {
    hipLaunchKernelGGL((decode_split_kernel<D, GH, EXACT>), dim3((unsigned)blocks), dim3(256), 0, st, p, a, pass);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL(decode_combine_kernel<D>, dim3(p.B * p.Hq), dim3(256), 0, st, p, a);
  return hipGetLastError();
}

template <int D, bool EXACT>
static hipError_t launch_split(const Problem &p, const DecodeArgs &a, hipStream_t st) {
  if (a.total_rows < 1) return hipErrorInvalidValue;
  if (!EXACT && p.g >= SEGATTN_DECODE_MFMA_MIN_G) {  // larger groups: the matrix-core form (segattn_decode_mfma.hip)
    const int resident = decode_mfma_resident(D);
    if (resident == 0) return hipErrorUnknown;
    DecodeArgs a2 = a;
    long long per = (a.total_rows + resident - 1) / resident;
    if (per < a.geom.decode_chunk) per = a.geom.decode_chunk;
    per = (per + 127) / 128 * 128;
    if (per > 0x7fffff00LL) return hipErrorInvalidValue;
    a2.rows_per_wg = (int)per;
    const hipError_t e = launch_decode_split_mfma(p, a2, (a.total_rows + per - 1) / per, st);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(decode_combine_kernel<D>, dim3(p.B * p.Hq), dim3(256), 0, st, p, a2);
    return hipGetLastError();
  }
  // heads per pass: the smallest of 1, 2, 4, 8 that covers the group (8 for larger groups)
  if (p.g > 4) return launch_split_gh<D, 8, EXACT>(p, a, st);
  if (p.g > 2) return launch_split_gh<D, 4, EXACT>(p, a, st);
  if (p.g == 2) return launch_split_gh<D, 2, EXACT>(p, a, st);
  return launch_split_gh<D, 1, EXACT>(p, a, st);
}

hipError_t launch_decode(const Problem &p, const DecodeArgs &a, int, hipStream_t st) {
  if (p.fp32_math) return p.D == 128 ? launch_split<128, true>(p, a, st) : launch_split<64, true>(p, a, st);
  return p.D == 128 ? launch_split<128, false>(p, a, st) : launch_split<64, false>(p, a, st);
}

}  // namespace segattn
