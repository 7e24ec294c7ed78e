// Backward of segment-level attention, validation kernels (fp32 FMA arithmetic, no MFMA) and the
// row statistic both backward paths share.
//
// Gradients of L = sum(O * dO) for O = softmax(scale Q K^T + M) V (Eq. 12 under the mask of
// Eq. 13), with gradient stopped where the paper stops it: every visible key contributes to dQ;
// dK and dV collect only the pairs inside a query's own segment or, for a head with the TAIL
// bit, its carried tail (the differentiable interface state of Sec. 3.2); rows reached only
// through the PAST bit are forward-only (no-gradient lemma, Appendix B).
//   P_ij = exp(scale q_i.k_j - LSE_i),  dP_ij = dO_i.v_j,  delta_i = dO_i.O_i,
//   dS_ij = P_ij (dP_ij - delta_i),  dQ_i = scale sum_j dS_ij k_j,
//   dK_j = scale sum_i dS_ij q_i,  dV_j = sum_i P_ij dO_i   (i over the differentiable pairs)
#include "segattn_internal.h"

namespace segattn {

__device__ inline float bf(unsigned short h) { return __uint_as_float((unsigned)h << 16); }

__device__ inline float wave_sum(float x) {
#pragma unroll
  for (int sh = 32; sh >= 1; sh >>= 1) x += __shfl_xor(x, sh);
  return x;
}

// delta[b,h,t] = sum_d dO[b,t,h,d] * O[b,t,h,d], and next to it nls = -lse / scale (the dK/dV
// kernel streams both per step as the starting values of its dP and score accumulators).  D/8 lanes
// per (row, head), 8 elements each.
template <int D>
__global__ __launch_bounds__(256) void bwd_delta_kernel(const Problem p, const BwdArgs a) {
  constexpr int LPR = D / 8;
  const long long item = ((long long)blockIdx.x * 256 + threadIdx.x) / LPR;  // (token row, h) flattened
  const int li = threadIdx.x % LPR;
  const long long tokens = a.cu_seqlens ? a.total : (long long)p.B * a.n;
  const long long items = tokens * p.Hq;
  float s = 0.f;
  if (item < items) {
    const uint4 g = *(const uint4 *)(a.dout + item * D + li * 8);
    const unsigned gw[4] = {g.x, g.y, g.z, g.w};
    if (p.out_fp32) {
      const float *o = (const float *)a.out + item * D + li * 8;
#pragma unroll
      for (int e = 0; e < 4; ++e)
        s += __uint_as_float(gw[e] << 16) * o[2 * e] + __uint_as_float(gw[e] & 0xffff0000u) * o[2 * e + 1];
    } else {
      const uint4 o = *(const uint4 *)((const unsigned short *)a.out + item * D + li * 8);
      const unsigned ow[4] = {o.x, o.y, o.z, o.w};
#pragma unroll
      for (int e = 0; e < 4; ++e)
        s += __uint_as_float(gw[e] << 16) * __uint_as_float(ow[e] << 16) +
             __uint_as_float(gw[e] & 0xffff0000u) * __uint_as_float(ow[e] & 0xffff0000u);
    }
  }
#pragma unroll
  for (int sh = 1; sh < LPR; sh <<= 1) s += __shfl_xor(s, sh);
  if (item < items && li == 0) {
    const long long bt = item / p.Hq;
    const int h = (int)(item % p.Hq);
    const SeqSpan sq = seq_span(p, a, seq_of_row(p, a, bt));
    const long long at = sq.stat0 + h * sq.stat_stride + (bt - sq.row0);
    a.delta[at] = s;
    a.nls[at] = -a.lse[at] / p.scale;
  }
}

// One wave per query row (b, t, h): lanes over d.
template <int D>
__global__ __launch_bounds__(256) void bwd_dq_fp32_kernel(const Problem p, const BwdArgs a) {
  constexpr int E = D / 64;
  const long long row = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  const long long tokens = a.cu_seqlens ? a.total : (long long)p.B * a.n;
  const long long rows = tokens * p.Hq;
  if (row >= rows) return;
  const int h = (int)(row % p.Hq);
  const long long bt = row / p.Hq;
  const SeqSpan sq = seq_span(p, a, seq_of_row(p, a, bt));
  const long long t = bt - sq.row0;
  const int kv = h / p.g, pol = p.policy[kv];
  const long long s0 = t / p.S * p.S;
  long long lo = s0;
  if (pol & SEGATTN_PAST) lo = 0;
  else if (pol & SEGATTN_TAIL) lo = s0 - p.T > 0 ? s0 - p.T : 0;
  float qv[E], gv[E], acc[E];
#pragma unroll
  for (int e = 0; e < E; ++e) {
    qv[e] = bf(a.q[row * D + lane * E + e]);
    gv[e] = bf(a.dout[row * D + lane * E + e]);
    acc[e] = 0.f;
  }
  const float lse = a.lse[sq.stat0 + h * sq.stat_stride + t];
  const float delta = a.delta[sq.stat0 + h * sq.stat_stride + t];
  for (long long j = lo; j <= t; ++j) {
    const unsigned short *kr = a.k + ((sq.row0 + j) * p.Hkv + kv) * D + lane * E;
    const unsigned short *vr = a.v + ((sq.row0 + j) * p.Hkv + kv) * D + lane * E;
    float kx[E], sd = 0.f, pd = 0.f;
#pragma unroll
    for (int e = 0; e < E; ++e) {
      kx[e] = bf(kr[e]);
      sd = fmaf(qv[e], kx[e], sd);
      pd = fmaf(gv[e], bf(vr[e]), pd);
    }
    sd = wave_sum(sd);
    pd = wave_sum(pd);
    const float pr = __expf(sd * p.scale - lse);
    const float ds = pr * (pd - delta);
#pragma unroll
    for (int e = 0; e < E; ++e) acc[e] = fmaf(ds, kx[e], acc[e]);
  }
#pragma unroll
  for (int e = 0; e < E; ++e) {
    const float r = acc[e] * p.scale;
    if (p.out_fp32) ((float *)a.dq)[row * D + lane * E + e] = r;
    else ((__bf16 *)a.dq)[row * D + lane * E + e] = (__bf16)r;
  }
}

// One wave per key row (b, j, kv): lanes over d; loops over the g query heads of the group and
// the queries whose pair with j is differentiable.
template <int D>
__global__ __launch_bounds__(256) void bwd_dkv_fp32_kernel(const Problem p, const BwdArgs a) {
  constexpr int E = D / 64;
  const long long row = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  const long long tokens = a.cu_seqlens ? a.total : (long long)p.B * a.n;
  const long long rows = tokens * p.Hkv;
  if (row >= rows) return;
  const int kv = (int)(row % p.Hkv), pol = p.policy[kv];
  const long long bj = row / p.Hkv;
  const SeqSpan sq = seq_span(p, a, seq_of_row(p, a, bj));
  const long long j = bj - sq.row0, n_b = sq.n;
  const long long s0 = j / p.S * p.S;
  const long long seg_end = s0 + p.S < n_b ? s0 + p.S : n_b;
  // queries of the next segment see j through the carried tail
  long long next_end = seg_end;
  if ((pol & SEGATTN_TAIL) && seg_end == s0 + p.S && j >= seg_end - p.T)
    next_end = seg_end + p.S < n_b ? seg_end + p.S : n_b;
  float kx[E], vx[E], dk[E], dv[E];
#pragma unroll
  for (int e = 0; e < E; ++e) {
    kx[e] = bf(a.k[row * D + lane * E + e]);
    vx[e] = bf(a.v[row * D + lane * E + e]);
    dk[e] = dv[e] = 0.f;
  }
  for (int hq = kv * p.g; hq < (kv + 1) * p.g; ++hq) {
    for (long long i = j; i < next_end; ++i) {
      const long long qrow = ((sq.row0 + i) * p.Hq + hq) * D + lane * E;
      float qx[E], gx[E], sd = 0.f, pd = 0.f;
#pragma unroll
      for (int e = 0; e < E; ++e) {
        qx[e] = bf(a.q[qrow + e]);
        gx[e] = bf(a.dout[qrow + e]);
        sd = fmaf(qx[e], kx[e], sd);
        pd = fmaf(gx[e], vx[e], pd);
      }
      sd = wave_sum(sd);
      pd = wave_sum(pd);
      const float pr = __expf(sd * p.scale - a.lse[sq.stat0 + hq * sq.stat_stride + i]);
      const float ds = pr * (pd - a.delta[sq.stat0 + hq * sq.stat_stride + i]);
#pragma unroll
      for (int e = 0; e < E; ++e) {
        dv[e] = fmaf(pr, gx[e], dv[e]);
        dk[e] = fmaf(ds, qx[e], dk[e]);
      }
    }
  }
#pragma unroll
  for (int e = 0; e < E; ++e) {
    const float rk = dk[e] * p.scale;
    if (p.out_fp32) {
      ((float *)a.dk)[row * D + lane * E + e] = rk;
      ((float *)a.dv)[row * D + lane * E + e] = dv[e];
    } else {
      ((__bf16 *)a.dk)[row * D + lane * E + e] = (__bf16)rk;
      ((__bf16 *)a.dv)[row * D + lane * E + e] = (__bf16)dv[e];
    }
  }
}

hipError_t launch_bwd_delta(const Problem &p, const BwdArgs &a, hipStream_t st) {
  const long long tokens = a.cu_seqlens ? a.total : (long long)p.B * a.n;
  const long long threads = tokens * p.Hq * (p.D / 8);
  const dim3 grid((unsigned)((threads + 255) / 256));
  if (p.D == 128) hipLaunchKernelGGL(bwd_delta_kernel<128>, grid, dim3(256), 0, st, p, a);
  else hipLaunchKernelGGL(bwd_delta_kernel<64>, grid, dim3(256), 0, st, p, a);
  return hipGetLastError();
}

hipError_t launch_bwd_fp32(const Problem &p, const BwdArgs &a, hipStream_t st) {
  const long long tokens = a.cu_seqlens ? a.total : (long long)p.B * a.n;
  const long long qrows = tokens * p.Hq, krows = tokens * p.Hkv;
  const dim3 gq((unsigned)((qrows + 3) / 4)), gk((unsigned)((krows + 3) / 4));
  if (p.D == 128) hipLaunchKernelGGL(bwd_dq_fp32_kernel<128>, gq, dim3(256), 0, st, p, a);
  else hipLaunchKernelGGL(bwd_dq_fp32_kernel<64>, gq, dim3(256), 0, st, p, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (p.D == 128) hipLaunchKernelGGL(bwd_dkv_fp32_kernel<128>, gk, dim3(256), 0, st, p, a);
  else hipLaunchKernelGGL(bwd_dkv_fp32_kernel<64>, gk, dim3(256), 0, st, p, a);
  return hipGetLastError();
}

}  // namespace segattn
