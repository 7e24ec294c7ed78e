// Bandwidth probe of libsegattn: the two access patterns of its HBM-bound kernels with nothing
// else in them, so that a benchmark can price those kernels against what the part sustains for
// the pattern rather than against the interface peak alone.
//   mode 0  read every 16-byte piece once (non-temporal, as the decode and retrieval scans read
//           their K/V rows); a checksum per workgroup keeps the loads alive
//   mode 1  read every 16-byte piece and write it back in place (as the in-place rotation does)
// and a clock probe: one sleeping wave per XCD that counts shader clocks against the constant-rate
// wall clock while other kernels run, which gives the clock the part holds under their load.
#include "segattn_internal.h"

namespace segattn {

typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
constexpr int kProbePieces = 8;  // 16-byte pieces per thread: a workgroup covers 32 KB

__global__ __launch_bounds__(256) void probe_read_kernel(const u32x4 *buf, long long pieces, unsigned *sink) {
  const long long base = (long long)blockIdx.x * (256 * kProbePieces) + threadIdx.x;
  u32x4 x[kProbePieces];
#pragma unroll
  for (int i = 0; i < kProbePieces; ++i) {
    const long long at = base + 256 * i;
    x[i] = at < pieces ? __builtin_nontemporal_load(buf + at) : u32x4{0u, 0u, 0u, 0u};
  }
  unsigned acc = 0;
#pragma unroll
  for (int i = 0; i < kProbePieces; ++i) acc ^= x[i][0] ^ x[i][1] ^ x[i][2] ^ x[i][3];
#pragma unroll
  for (int sh = 32; sh >= 1; sh >>= 1) acc ^= __shfl_xor(acc, sh);
  if ((threadIdx.x & 63) == 0 && acc == 0x9e3779b9u) sink[0] = acc;  // practically never taken: no store traffic
}

template <int PIECES>
__global__ __launch_bounds__(256) void probe_rmw_kernel(u32x4 *buf, long long pieces) {
  const long long base = (long long)blockIdx.x * (256 * PIECES) + threadIdx.x;
  u32x4 x[PIECES];
#pragma unroll
  for (int i = 0; i < PIECES; ++i) {
    const long long at = base + 256 * i;
    if (at < pieces) x[i] = buf[at];
  }
#pragma unroll
  for (int i = 0; i < PIECES; ++i) {
    const long long at = base + 256 * i;
    if (at < pieces) {
      x[i][0] ^= 0x80008000u;  // flips two sign bits: two probes restore the buffer
      buf[at] = x[i];
    }
  }
}

// One wave per workgroup, eight workgroups (the dispatcher deals them to the eight XCDs in turn).
// Each sleeps until `ticks` of the wall clock have passed, a bound every wave reaches, and then
// stores the shader clocks and wall ticks it saw.
__global__ __launch_bounds__(64) void clock_probe_kernel(unsigned long long ticks, unsigned long long *out) {
  const unsigned long long t0 = __builtin_amdgcn_s_memrealtime();
  const unsigned long long c0 = __builtin_readcyclecounter();
  unsigned long long t;
  do {
    __builtin_amdgcn_s_sleep(127);
    t = __builtin_amdgcn_s_memrealtime();
  } while (t - t0 < ticks);
  const unsigned long long c1 = __builtin_readcyclecounter();
  if (threadIdx.x == 0) {
    out[2 * blockIdx.x] = c1 - c0;
    out[2 * blockIdx.x + 1] = t - t0;
  }
}

hipError_t launch_clock_probe(unsigned long long ticks, unsigned long long *out, hipStream_t st) {
  hipLaunchKernelGGL(clock_probe_kernel, dim3(kClockProbeWaves), dim3(64), 0, st, ticks, out);
  return hipGetLastError();
}

// Matrix-pipe ceiling: every wave runs eight independent accumulation chains of
// v_mfma_f32_32x32x16_bf16 from registers and touches no memory in the loop, so the launch shows
// the dense bf16 rate the part reaches (and, with the clock probe beside it, the clock it holds)
// when nothing but the matrix pipes is busy.  The part is power-limited: with random operands it
// holds a much lower clock than with constant ones.
typedef __bf16 probe_bf16x8 __attribute__((ext_vector_type(8)));
typedef float probe_f32x16 __attribute__((ext_vector_type(16)));
constexpr int kMfmaProbeChains = 8;
// distinct (A, B) operand pairs the chains rotate through: with one pair every product repeats, with
// eight the operand fetch, not the pipe, sets the pace (85 % even with constant operands); four keep
// the pipes 99 % busy
constexpr int kMfmaProbeOperandSets = 4;
template <int SETS>
__global__ __launch_bounds__(256) void probe_mfma_kernel(int iters, int quiet, unsigned seed, float *sink) {
  // operands: pseudo-random bf16 in [-1, 1), different for every lane, register and chain; with
  // `quiet` every operand element is the same constant instead (such products switch almost no
  // wires, draw far less power and run at a higher clock than products of real data)
  unsigned h = seed ^ (threadIdx.x * 2654435761u) ^ (blockIdx.x * 40503u);
  auto next = [&]() {
    h = h * 1664525u + 1013904223u;
    return quiet ? (__bf16)0.00390625f : (__bf16)((float)(int)(h >> 8) * (1.0f / 8388608.0f) - 1.0f);
  };
  probe_bf16x8 a[SETS], b[SETS];
#pragma unroll
  for (int c = 0; c < SETS; ++c)
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      a[c][i] = next();
      b[c][i] = next();
    }
  probe_f32x16 acc[kMfmaProbeChains];
#pragma unroll
  for (int c = 0; c < kMfmaProbeChains; ++c)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[c][r] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int c = 0; c < kMfmaProbeChains; ++c)
      acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[c % SETS], b[c % SETS], acc[c], 0, 0, 0);
  }
  float total = 0.f;
#pragma unroll
  for (int c = 0; c < kMfmaProbeChains; ++c)
#pragma unroll
    for (int r = 0; r < 16; ++r) total += acc[c][r];
  if (total == -1.2345678e30f) sink[0] = total;  // practically never: keeps the chains alive, no store traffic
}

hipError_t launch_mfma_probe(int iters, int quiet, int workgroups, float *sink, hipStream_t st) {
  hipLaunchKernelGGL(probe_mfma_kernel<kMfmaProbeOperandSets>, dim3((unsigned)workgroups), dim3(256), 0, st, iters, quiet,
                     0x9e3779b9u, sink);
  return hipGetLastError();
}

hipError_t launch_probe(void *buf, long long bytes, int mode, void *sink, hipStream_t st) {
  const long long pieces = bytes / 16;
  const long long blocks = (pieces + 256 * kProbePieces - 1) / (256 * kProbePieces);
  if (blocks <= 0 || blocks > 0x7fffffffLL) return hipErrorInvalidValue;
  if (mode == 0) {
    hipLaunchKernelGGL(probe_read_kernel, dim3((unsigned)blocks), dim3(256), 0, st, (const u32x4 *)buf, pieces, (unsigned *)sink);
  } else {
    // two pieces per thread: more in flight per thread measured slower (5.7 TB/s against 5.5 with one
    // or four and 4.2 with eight)
    const long long b2 = (pieces + 256 * 2 - 1) / (256 * 2);
    if (b2 > 0x7fffffffLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL(probe_rmw_kernel<2>, dim3((unsigned)b2), dim3(256), 0, st, (u32x4 *)buf, pieces);
  }
  return hipGetLastError();
}

}  // namespace segattn
