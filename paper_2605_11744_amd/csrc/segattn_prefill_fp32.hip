// fp32 validation kernel of libsegattn's prefill: the same work decomposition and key ranges
// as the MFMA kernel, plain fp32 FMA arithmetic, fp32 output (Eq. 12 / Eq. 13, Appendix C).
#include "segattn_work.h"

namespace segattn {

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

hipError_t launch_prefill_fp32(const Problem &p, const PrefillArgs &a, long long grid, hipStream_t st) {
  if (p.D == 128) hipLaunchKernelGGL(prefill_fp32_kernel<128>, dim3((unsigned)grid), dim3(256), 0, st, p, a);
  else hipLaunchKernelGGL(prefill_fp32_kernel<64>, dim3((unsigned)grid), dim3(256), 0, st, p, a);
  return hipGetLastError();
}

}  // namespace segattn
