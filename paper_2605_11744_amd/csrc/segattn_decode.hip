// Decode path of libsegattn: one new token per sequence attends over the visible window
// [prefix | open segment] of every KV head (Eq. 12 / Eq. 13 for a single query row; Eq. 2's
// conditioning on x_<t, C_{i-1}, R_{i-1}).  The work is HBM-bound (every visible K and V row
// is read once per KV head and serves the g query heads of the group), so it is a split-K
// reduction:
//   decode_split_kernel    grid (split, b*Hkv): a workgroup streams one chunk of the window
//                          with 16-byte coalesced loads (D/8 lanes per key row), forms the g
//                          dot products per row with a DPP reduction inside each lane group,
//                          keeps an online-softmax state per lane group, merges the groups
//                          with wave shuffles and the four waves through LDS, and writes one
//                          partial (m, l, acc[D]) per query head.
//   decode_combine_kernel  one wave per (b, query head): merges the partials of all splits.
#include "segattn_internal.h"

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

template <int D, int GH>
__global__ __launch_bounds__(256) void decode_split_kernel(const Problem p, const DecodeArgs a,
                                                          const int head_pass) {
  constexpr int LPR = D / 8;        // lanes per key row
  constexpr int GPW = 64 / LPR;     // key rows per wave-wide load
  constexpr int U = 4;              // rows in flight per lane group
  const int b = blockIdx.y / p.Hkv, kv = blockIdx.y % p.Hkv;
  const int *meta = meta_ro(a.cache, a.geom, p, b, kv);
  int lo, seg_row0;
  window_of(p, kv, meta, lo, seg_row0);
  const int hi = seg_row0 + meta[META_FILL];
  const int c0 = lo + blockIdx.x * a.geom.decode_chunk;
  if (c0 >= hi) return;
  const int c1 = min(hi, c0 + a.geom.decode_chunk);

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int grp = lane / LPR, li = lane % LPR;
  const int head0 = kv * p.g + head_pass * GH;
  const float c = p.scale_log2e;

  float qf[GH][8];
#pragma unroll
  for (int h = 0; h < GH; ++h)
    unpack8(*(const uint4 *)(a.q + ((long long)b * p.Hq + head0 + h) * D + li * 8), qf[h]);

  float m_run[GH], l_run[GH], acc[GH][8];
#pragma unroll
  for (int h = 0; h < GH; ++h) {
    m_run[h] = -INFINITY;
    l_run[h] = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[h][e] = 0.f;
  }

  const uint4 *kb = (const uint4 *)(a.cache + k_block_off(p, a.geom, b, kv)) + li;
  const uint4 *vb = (const uint4 *)(a.cache + v_block_off(p, a.geom, b, kv)) + li;
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
      unpack8(kr[u], kf);
#pragma unroll
      for (int h = 0; h < GH; ++h) {
        float d = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) d = fmaf(qf[h][e], kf[e], d);
        d = group_sum<LPR>(d);
        s[u][h] = row[u] < c1 ? d : -INFINITY;
      }
    }
    if (row[0] >= c1) continue;  // whole lane group past the end (rows ascend with u)
    float pw[U][GH];
#pragma unroll
    for (int h = 0; h < GH; ++h) {
      float mx = m_run[h];
#pragma unroll
      for (int u = 0; u < U; ++u) mx = fmaxf(mx, s[u][h]);
      const float alpha = __builtin_amdgcn_exp2f((m_run[h] - mx) * c);
      const float mc = mx * c;
      float ps = 0.f;
#pragma unroll
      for (int u = 0; u < U; ++u) {
        pw[u][h] = __builtin_amdgcn_exp2f(fmaf(s[u][h], c, -mc));
        ps += pw[u][h];
      }
      l_run[h] = l_run[h] * alpha + ps;
      m_run[h] = mx;
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[h][e] *= alpha;
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      float vf[8];
      unpack8(vr[u], vf);
#pragma unroll
      for (int h = 0; h < GH; ++h)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[h][e] = fmaf(pw[u][h], vf[e], acc[h][e]);
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
    float *slot = ws + (ws_slot_base(p, a.geom, b, head0 + h) + blockIdx.x) * (2 + D);
    if (d == 0) {
      slot[0] = mx;
      slot[1] = l;
    }
    slot[2 + d] = o;
  }
}

template <int D>
__global__ __launch_bounds__(64) void decode_combine_kernel(const Problem p, const DecodeArgs a) {
  const int b = blockIdx.x / p.Hq, head = blockIdx.x % p.Hq;
  const int kv = head / p.g;
  const int *meta = meta_ro(a.cache, a.geom, p, b, kv);
  int lo, seg_row0;
  window_of(p, kv, meta, lo, seg_row0);
  const int hi = seg_row0 + meta[META_FILL];
  const int ns = (hi - lo + a.geom.decode_chunk - 1) / a.geom.decode_chunk;
  const float *ws = (const float *)(a.cache + a.geom.ws_off) + ws_slot_base(p, a.geom, b, head) * (2 + D);
  const int lane = threadIdx.x;
  const float c = p.scale_log2e;
  // global max and denominator: lanes stride over the splits, then a wave reduction
  float mx = -INFINITY;
  for (int s = lane; s < ns; s += 64) mx = fmaxf(mx, ws[(long long)s * (2 + D)]);
#pragma unroll
  for (int sh = 1; sh < 64; sh <<= 1) mx = fmaxf(mx, __shfl_xor(mx, sh));
  float l = 0.f;
  for (int s = lane; s < ns; s += 64) {
    const float *slot = ws + (long long)s * (2 + D);
    l += slot[1] * __builtin_amdgcn_exp2f((slot[0] - mx) * c);
  }
#pragma unroll
  for (int sh = 1; sh < 64; sh <<= 1) l += __shfl_xor(l, sh);
  constexpr int DPL = D / 64;
  float o[DPL];
#pragma unroll
  for (int e = 0; e < DPL; ++e) o[e] = 0.f;
  for (int s = 0; s < ns; ++s) {
    const float *slot = ws + (long long)s * (2 + D);
    const float wgt = __builtin_amdgcn_exp2f((slot[0] - mx) * c);
#pragma unroll
    for (int e = 0; e < DPL; ++e) o[e] = fmaf(slot[2 + lane * DPL + e], wgt, o[e]);
  }
  const float inv = 1.f / l;
  const long long obase = ((long long)b * p.Hq + head) * D + lane * DPL;
#pragma unroll
  for (int e = 0; e < DPL; ++e) {
    if (p.out_fp32) ((float *)a.out)[obase + e] = o[e] * inv;
    else ((__bf16 *)a.out)[obase + e] = (__bf16)(o[e] * inv);
  }
  if (lane == 0) a.lse[(long long)b * p.Hq + head] = mx * p.scale + __logf(l);
}

template <int D>
static hipError_t launch_split(const Problem &p, const DecodeArgs &a, hipStream_t st) {
  const dim3 grid(a.max_splits, p.B * p.Hkv);
  int gh = (p.g % 4 == 0) ? 4 : (p.g % 2 == 0) ? 2 : 1;
  for (int pass = 0; pass < p.g / gh; ++pass) {
    if (gh == 4) hipLaunchKernelGGL((decode_split_kernel<D, 4>), grid, dim3(256), 0, st, p, a, pass);
    else if (gh == 2) hipLaunchKernelGGL((decode_split_kernel<D, 2>), grid, dim3(256), 0, st, p, a, pass);
    else hipLaunchKernelGGL((decode_split_kernel<D, 1>), grid, dim3(256), 0, st, p, a, pass);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL(decode_combine_kernel<D>, dim3(p.B * p.Hq), dim3(64), 0, st, p, a);
  return hipGetLastError();
}

hipError_t launch_decode(const Problem &p, const DecodeArgs &a, int, hipStream_t st) {
  return p.D == 128 ? launch_split<128>(p, a, st) : launch_split<64>(p, a, st);
}

}  // namespace segattn
