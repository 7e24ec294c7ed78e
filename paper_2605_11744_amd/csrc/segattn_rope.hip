// RoPE for segmented execution (Sec. 3.4 "RoPE Re-indexing for Prefix Concatenation",
// Appendix E).  The paper gives a prefix of length P the key positions 0..P-1 and the segment's
// queries and keys the positions P..P+m-1.  Standard RoPE scores depend on position differences
// only, so for a prefix that is a contiguous run of tokens ending at the segment start (the
// carried tail, the whole history) this is the same as rotating every token once by its
// absolute position -- which is what rope_apply_kernel does, in place, before the rows are
// attended to and committed.  A retrieved prefix is not contiguous: its rows are turned to the
// positions s-R .. s-1 just before the segment when they are gathered (cache_select_kernel).
//
// Channel pair (i, i + D/2) is turned by position * theta^(-2i/D).  The angle is formed and
// reduced to [-pi, pi] in double precision (a float product is off by up to 0.01 rad at
// position 10^5), sine and cosine are single precision.  HBM-bound: every element is read and
// written once.
#include <math.h>

#include "segattn_internal.h"

namespace segattn {

// sine and cosine of pos * inv_freq, the angle reduced to [-pi, pi] in double precision
__device__ inline void rope_sincos(double pos, double inv_freq, float &sn, float &cs) {
  const double a = pos * inv_freq;
  const double two_pi = 6.283185307179586476925286766559, inv_two_pi = 0.15915494309189533576888376337251;
  const float r = (float)(a - two_pi * rint(a * inv_two_pi));
  sincosf(r, &sn, &cs);
}

// Rotate 8 consecutive channels (lo) with their partners D/2 further on (hi).
__device__ inline void rope_rotate8(uint4 &lo, uint4 &hi, const float (&sn)[8], const float (&cs)[8]) {
  unsigned *lw = (unsigned *)&lo, *hw = (unsigned *)&hi;
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    unsigned lo_out = 0, hi_out = 0;
#pragma unroll
    for (int e = 0; e < 2; ++e) {
      const float a = __uint_as_float(e ? (lw[w] & 0xffff0000u) : (lw[w] << 16));
      const float b = __uint_as_float(e ? (hw[w] & 0xffff0000u) : (hw[w] << 16));
      const __bf16 ya = (__bf16)(a * cs[2 * w + e] - b * sn[2 * w + e]);
      const __bf16 yb = (__bf16)(a * sn[2 * w + e] + b * cs[2 * w + e]);
      lo_out |= (unsigned)__builtin_bit_cast(unsigned short, ya) << (16 * e);
      hi_out |= (unsigned)__builtin_bit_cast(unsigned short, yb) << (16 * e);
    }
    lw[w] = lo_out;
    hw[w] = hi_out;
  }
}

// One thread per (b, row, group of 8 channel pairs): the angles depend on the position and the
// channel only, so the thread forms its 8 sines and cosines once and walks over all heads of q
// and k with them.
template <int D>
__global__ __launch_bounds__(256) void rope_apply_kernel(const Problem p, const RopeArgs a) {
  constexpr int LPH = D / 16;  // threads per row
  const long long t = (long long)blockIdx.x * 256 + threadIdx.x;
  const int li = (int)(t % LPH);
  const long long br = t / LPH;  // (b, row)
  if (br >= (long long)p.B * a.rows) return;
  const long long b = br / a.rows, r = br % a.rows;
  const double pos = (double)((a.pos0 ? a.pos0[b] : 0) + r);
  float sn[8], cs[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) rope_sincos(pos, a.inv_freq[8 * li + e], sn[e], cs[e]);
  unsigned short *qrow = a.q + br * p.Hq * D + 8 * li;
#pragma unroll 4
  for (int h = 0; h < p.Hq; ++h, qrow += D) {
    uint4 lo = *(const uint4 *)qrow, hi = *(const uint4 *)(qrow + D / 2);
    rope_rotate8(lo, hi, sn, cs);
    *(uint4 *)qrow = lo;
    *(uint4 *)(qrow + D / 2) = hi;
  }
  unsigned short *krow = a.k + br * p.Hkv * D + 8 * li;
#pragma unroll 4
  for (int h = 0; h < p.Hkv; ++h, krow += D) {
    uint4 lo = *(const uint4 *)krow, hi = *(const uint4 *)(krow + D / 2);
    rope_rotate8(lo, hi, sn, cs);
    *(uint4 *)krow = lo;
    *(uint4 *)(krow + D / 2) = hi;
  }
}

hipError_t launch_rope_apply(const Problem &p, const RopeArgs &a, hipStream_t st) {
  const long long threads = (long long)p.B * a.rows * (p.D / 16);
  const long long blocks = (threads + 255) / 256;
  if (blocks <= 0 || blocks > 0x7fffffffLL) return hipErrorInvalidValue;
  if (p.D == 128) hipLaunchKernelGGL(rope_apply_kernel<128>, dim3((unsigned)blocks), dim3(256), 0, st, p, a);
  else hipLaunchKernelGGL(rope_apply_kernel<64>, dim3((unsigned)blocks), dim3(256), 0, st, p, a);
  return hipGetLastError();
}

}  // namespace segattn
