// Decode path of libsegattn: one new token per sequence attends over the visible window
// [prefix | open segment] of every KV head (Eq. 12 / Eq. 13 for a single query row; Eq. 2's
// conditioning on x_<t, C_{i-1}, R_{i-1}).  The work is HBM-bound (every visible K and V row
// is read once per KV head and serves the g query heads of the group), so it is a split-K
// reduction:
//   decode_split_kernel    one workgroup per (b, KV head, chunk of the window): it streams the chunk
//                          with 16-byte coalesced loads (D/8 lanes per key row), forms the g
//                          dot products per row with a DPP reduction inside each lane group,
//                          keeps an online-softmax state per lane group, merges the groups
//                          with wave shuffles and the four waves through LDS, and writes one
//                          partial (m, l, acc[D]) per query head.
//   decode_combine_kernel  one workgroup per (b, query head): merges the partials of all splits.
#include "segattn_internal.h"

#ifndef SEGATTN_DECODE_U
#define SEGATTN_DECODE_U 8
#endif

namespace segattn {

__device__ inline const int *meta_ro(const unsigned char *cache, const CacheGeom &g, const Problem &p, int b,
                                     int h) {
  return (const int *)(cache + g.meta_off) + ((long long)b * p.Hkv + h) * kMetaInts;
}

// floats of split-K workspace before (b, query head): partial slots are (2 + D) floats
__device__ inline long long ws_slot_base(const Problem &p, const CacheGeom &g, int b, int head) {
  const int kv = head / p.g;
  const long long np = p.past_before[kv];
  const long long per_seq = (long long)p.g * ((long long)p.n_past * g.ws_splits_past +
                                              (long long)(p.Hkv - p.n_past) * g.ws_splits_other);
  const long long before = (long long)p.g * (np * g.ws_splits_past + (kv - np) * g.ws_splits_other);
  const long long mine = (p.policy[kv] & SEGATTN_PAST) ? g.ws_splits_past : g.ws_splits_other;
  return (long long)b * per_seq + before + (long long)(head % p.g) * mine;
}

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

__device__ inline float dot2_bf16(unsigned a, unsigned b, float c) {  // a.lo*b.lo + a.hi*b.hi + c
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, a), __builtin_bit_cast(bf16x2, b), c, false);
}

// blockIdx.x -> (split, b, kv): PAST heads first (they have up to splits_past splits), then the
// others (at most splits_other), so that few workgroups find nothing to do.
__device__ inline bool decode_block(const Problem &p, const DecodeArgs &a, int bid, int &split, int &b, int &kv) {
  const int past_blocks = p.B * p.n_past * a.splits_past;
  int hidx;
  if (bid < past_blocks) {
    split = bid % a.splits_past;
    const int r = bid / a.splits_past;
    hidx = r % p.n_past;
    b = r / p.n_past;
  } else {
    const int y = bid - past_blocks;
    const int n_other = p.Hkv - p.n_past;
    split = y % a.splits_other;
    const int r = y / a.splits_other;
    hidx = p.n_past + r % n_other;
    b = r / n_other;
  }
  kv = p.order[hidx];
  return true;
}

// EXACT: fp32 weights and fp32 FMAs throughout (validation mode).  Otherwise the dot products
// use v_dot2_f32_bf16 on the bf16 pairs as they come from memory, and the weights are rounded to
// bf16 for the PV product (as in the prefill kernel; the row sums use the same rounded values).
template <int D, int GH, bool EXACT>
__global__ __launch_bounds__(256) void decode_split_kernel(const Problem p, const DecodeArgs a,
                                                          const int head_pass) {
  constexpr int LPR = D / 8;        // lanes per key row
  constexpr int GPW = 64 / LPR;     // key rows per wave-wide load
  constexpr int U = SEGATTN_DECODE_U;  // rows in flight per lane group
  int split, b, kv;
  decode_block(p, a, blockIdx.x, split, b, kv);
  const int *meta = meta_ro(a.cache, a.geom, p, b, kv);
  int lo, seg_row0;
  window_of(p, a.geom, kv, meta, lo, seg_row0);
  const int hi = seg_row0 + meta[META_FILL];
  const int c0 = lo + split * a.geom.decode_chunk;
  if (c0 >= hi) return;
  const int c1 = min(hi, c0 + a.geom.decode_chunk);

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int grp = lane / LPR, li = lane % LPR;
  const int head0 = kv * p.g + head_pass * GH;
  const float c = p.scale_log2e;

  uint4 qp[GH];   // this lane's 8 query elements per head, as bf16 pairs
  float qf[EXACT ? GH : 1][8];
#pragma unroll
  for (int h = 0; h < GH; ++h) {
    qp[h] = *(const uint4 *)(a.q + ((long long)b * p.Hq + head0 + h) * D + li * 8);
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
      kr[u] = kb[(long long)rc * LPR];
      vr[u] = vb[(long long)rc * LPR];
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

  // ---- merge the lane groups of a wave (shuffles), then the four waves (LDS)
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
  __shared__ float sm_m[4][GH], sm_l[4][GH], sm_acc[4][GH][D];
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
  float *ws = (float *)(a.cache + a.geom.ws_off);
  for (int idx = tid; idx < GH * D; idx += 256) {
    const int h = idx / D, d = idx % D;
    float mx = -INFINITY;
#pragma unroll
    for (int w = 0; w < 4; ++w) mx = fmaxf(mx, sm_m[w][h]);
    float l = 0.f, o = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const float wgt = (sm_m[w][h] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f((sm_m[w][h] - mx) * c);
      l += sm_l[w][h] * wgt;
      o += sm_acc[w][h][d] * wgt;
    }
    float *slot = ws + (ws_slot_base(p, a.geom, b, head0 + h) + split) * (2 + D);
    if (d == 0) {
      slot[0] = mx;
      slot[1] = l;
    }
    slot[2 + d] = o;
  }
}

// One workgroup per (b, query head).  All threads find the global maximum over the splits; then
// wave w accumulates the splits congruent to w mod 4 (lanes over the D outputs) and the four
// partial sums meet in LDS.
template <int D>
__global__ __launch_bounds__(256) void decode_combine_kernel(const Problem p, const DecodeArgs a) {
  const int b = blockIdx.x / p.Hq, head = blockIdx.x % p.Hq;
  const int kv = head / p.g;
  const int *meta = meta_ro(a.cache, a.geom, p, b, kv);
  int lo, seg_row0;
  window_of(p, a.geom, kv, meta, lo, seg_row0);
  const int hi = seg_row0 + meta[META_FILL];
  const int ns = (hi - lo + a.geom.decode_chunk - 1) / a.geom.decode_chunk;
  const float *ws = (const float *)(a.cache + a.geom.ws_off) + ws_slot_base(p, a.geom, b, head) * (2 + D);
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const float c = p.scale_log2e;
  constexpr int DPL = D / 64;
  __shared__ float sm_max[4], sm_l[4], sm_o[4][D];

  float mx = -INFINITY;
  for (int s = tid; s < ns; s += 256) mx = fmaxf(mx, ws[(long long)s * (2 + D)]);
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
    const float *slot = ws + (long long)s * (2 + D);
    const float wgt = __builtin_amdgcn_exp2f((slot[0] - mx) * c);
    l = fmaf(slot[1], wgt, l);
#pragma unroll
    for (int e = 0; e < DPL; ++e) o[e] = fmaf(slot[2 + lane * DPL + e], wgt, o[e]);
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

template <int D, bool EXACT>
static hipError_t launch_split(const Problem &p, const DecodeArgs &a, hipStream_t st) {
  const long long blocks = (long long)p.B * ((long long)p.n_past * a.splits_past +
                                             (long long)(p.Hkv - p.n_past) * a.splits_other);
  const dim3 grid((unsigned)blocks);
  int gh = (p.g % 4 == 0) ? 4 : (p.g % 2 == 0) ? 2 : 1;
  for (int pass = 0; pass < p.g / gh; ++pass) {
    if (gh == 4) hipLaunchKernelGGL((decode_split_kernel<D, 4, EXACT>), grid, dim3(256), 0, st, p, a, pass);
    else if (gh == 2) hipLaunchKernelGGL((decode_split_kernel<D, 2, EXACT>), grid, dim3(256), 0, st, p, a, pass);
    else hipLaunchKernelGGL((decode_split_kernel<D, 1, EXACT>), grid, dim3(256), 0, st, p, a, pass);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL(decode_combine_kernel<D>, dim3(p.B * p.Hq), dim3(256), 0, st, p, a);
  return hipGetLastError();
}

hipError_t launch_decode(const Problem &p, const DecodeArgs &a, int, hipStream_t st) {
  if (p.fp32_math) return p.D == 128 ? launch_split<128, true>(p, a, st) : launch_split<64, true>(p, a, st);
  return p.D == 128 ? launch_split<128, false>(p, a, st) : launch_split<64, false>(p, a, st);
}

}  // namespace segattn
