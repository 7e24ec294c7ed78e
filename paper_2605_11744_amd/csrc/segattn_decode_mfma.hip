// Decode split kernel on the matrix cores (the bf16 path of seg_attn_decode).
//
// The g query heads of a GQA group are the columns of one 32-column operand (16 per pass: what the
// merge area inside the tiles holds; a group of up to 16 heads streams its K/V rows once): per tile
// of 32 key rows a wave forms
//   S^T[key][head] = K_tile . Q^T       v_mfma_f32_32x32x16_bf16, A = K rows, B = Q^T (registers)
//   P = exp2(S^T c - m c)               online softmax per head (lane = head)
//   O^T[d][head] += V_tile^T . P^T      A = V^T via ds_read_b64_tr_b16, B = P from the S^T registers
// exactly as the prefill kernel does for 32 query rows.  The products are nearly free here (the
// work is HBM-bound); what they buy is a softmax of 16 elements per lane and tile instead of a
// dot-product-and-reduce pass per row and head: a group of eight heads runs as fast as a group
// of one (the vector-ALU form in segattn_decode.hip needs ~150 instructions per row and lane
// group for eight heads and is bound by them).  Same slices of the concatenated windows, same
// partials (acc[D], m, l) and the same combine kernel as that form.  A wave owns every fourth tile
// of the slice; tiles go HBM -> registers (one tile ahead) -> a wave-private LDS tile with the
// prefill kernel's chunk swizzles -> operands, so the loop needs no barrier.
#include "segattn_decode_slices.h"

namespace segattn {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
#define LDS_AS __attribute__((address_space(3)))

constexpr int kDecTile = 32;   // key rows per tile
constexpr int kDecHeads = 16;  // query heads per pass (columns in use of the 32-column operand)

__device__ inline float dec_half_max(float x) {  // max over lanes l and l^32
  const int xi = __float_as_int(x);
  const auto sw = __builtin_amdgcn_permlane32_swap(xi, xi, false, false);
  return fmaxf(__int_as_float(sw[0]), __int_as_float(sw[1]));
}
__device__ inline float dec_half_sum(float x) {
  const int xi = __float_as_int(x);
  const auto sw = __builtin_amdgcn_permlane32_swap(xi, xi, false, false);
  return __int_as_float(sw[0]) + __int_as_float(sw[1]);
}

template <int D>
__global__ __launch_bounds__(256, 2) void decode_split_mfma_kernel(const Problem p, const DecodeArgs a,
                                                                   const int head_pass) {
  constexpr int NC = D / 16, NB = D / 32;
  constexpr int kRowBytes = 2 * D, kChunks = D / 8, kTileBytes = kDecTile * kRowBytes;
  constexpr int kRowsPer256 = 256 / kRowBytes;   // rows sharing one 64-bank window (1 or 2)
  constexpr int RPL = 1024 / kRowBytes;          // rows per 1 KB wave load
  constexpr int NL = kDecTile / RPL;             // loads per tile and tensor
  auto swz_k = [](int row) { return (row / kRowsPer256) & 7; };
  auto swz_v = [](int row) { return 4 * ((row / kRowsPer256) % (kChunks / 4)); };

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int hi = lane >> 5, col = lane & 31;
  const int i16 = lane & 15, g16 = (lane >> 4) & 1;
  const float c = p.scale_log2e;

  // [K tile | V tile] per wave; the merge of the four waves at the end of a window reuses it
  __shared__ __attribute__((aligned(1024))) unsigned char tiles[4][2 * kTileBytes];
  static_assert(4 * 2 * kTileBytes >= (int)sizeof(float) * 4 * kDecHeads * (D + 2), "merge area fits the tiles");

  // ---- where this workgroup's slice begins
  const int n_win = p.B * p.Hkv;
  const long long start = (long long)blockIdx.x * a.rows_per_wg;
  int w, off;
  decode_slice_start(p, a, start, w, off);
  if (w < 0) return;
  int split = (int)((long long)blockIdx.x - (start - off) / a.rows_per_wg);
  int remaining = a.rows_per_wg;
  int *counts = ws_counts(a.cache, a.geom);
  float *slots = ws_slots(a.cache, a.geom, p);

  unsigned char *tile = tiles[wave];
  // operand read offsets inside the wave's tile pair (the prefill kernel's layouts)
  int koff[NC];
#pragma unroll
  for (int kc = 0; kc < NC; ++kc) koff[kc] = col * kRowBytes + (((2 * kc + hi) ^ swz_k(col)) << 4);
  int voff[NB];
  {
    const int vrow = 4 * hi + (i16 >> 2);
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      const int chunk = 4 * nb + 2 * g16 + ((i16 & 3) >> 1);
      voff[nb] = kTileBytes + vrow * kRowBytes + ((chunk ^ swz_v(vrow)) << 4) + 8 * (i16 & 1);
    }
  }
  // where this lane's 16-byte pieces of a tile land (load i: row RPL i + lane / chunks)
  int st_k[NL], st_v[NL];
#pragma unroll
  for (int i = 0; i < NL; ++i) {
    const int r = RPL * i + lane / kChunks, ch = lane % kChunks;
    st_k[i] = r * kRowBytes + ((ch ^ swz_k(r)) << 4);
    st_v[i] = kTileBytes + r * kRowBytes + ((ch ^ swz_v(r)) << 4);
  }

  for (; remaining > 0 && w < n_win; ++w, off = 0, split = 0) {
    const int b = w / p.Hkv, kv = w % p.Hkv;
    int lo, hi_;
    decode_window_rows(p, a, w, lo, hi_);
    lo = __builtin_amdgcn_readfirstlane(lo);
    hi_ = __builtin_amdgcn_readfirstlane(hi_);
    const int c0 = lo + off;
    const int c1 = min(hi_, c0 + remaining);
    if (c1 <= c0) continue;
    remaining -= c1 - c0;
    const int head0 = kv * p.g + head_pass * kDecHeads;
    const int live = min(kDecHeads, p.g - head_pass * kDecHeads);

    // Q^T: column col = head head0 + col (zero beyond the live heads)
    bf16x8 Qr[NC];
    {
      const unsigned short *qrow = a.q + ((long long)b * p.Hq + head0 + (col < live ? col : 0)) * D + 8 * hi;
#pragma unroll
      for (int kc = 0; kc < NC; ++kc) {
        u32x4 x = *(const u32x4 *)(qrow + 16 * kc);
        if (col >= live) x = u32x4{0u, 0u, 0u, 0u};
        Qr[kc] = __builtin_bit_cast(bf16x8, x);
      }
    }
    f32x16 O[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
      for (int r = 0; r < 16; ++r) O[nb][r] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;

    const unsigned char *kb = a.cache + attn_k_off(p, a.geom, b, kv);
    const unsigned char *vb = a.cache + attn_v_off(p, a.geom, b, kv);
    u32x4 nk[NL], nv[NL];  // the wave's next tile, in flight
    auto fetch = [&](int r0) __attribute__((always_inline)) {
#pragma unroll
      for (int i = 0; i < NL; ++i) {
        int r = r0 + RPL * i + lane / kChunks;
        r = r < c1 ? r : c1 - 1;  // clamp: stays inside the window
        const long long o = (long long)r * kRowBytes + (lane % kChunks) * 16;
        nk[i] = __builtin_nontemporal_load((const u32x4 *)(kb + o));
        nv[i] = __builtin_nontemporal_load((const u32x4 *)(vb + o));
      }
    };
    const int first = c0 + kDecTile * wave;
    if (first < c1) fetch(first);
    for (int r0 = first; r0 < c1; r0 += 4 * kDecTile) {
#pragma unroll
      for (int i = 0; i < NL; ++i) {
        *(u32x4 *)(tile + st_k[i]) = nk[i];
        *(u32x4 *)(tile + st_v[i]) = nv[i];
      }
      if (r0 + 4 * kDecTile < c1) fetch(r0 + 4 * kDecTile);
      // S^T
      f32x16 S = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int kc = 0; kc < NC; ++kc) {
        const bf16x8 ka = *(const bf16x8 *)(tile + koff[kc]);
        S = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, Qr[kc], S, 0, 0, 0);
      }
      // rows past the end of the window's part: register r of the lane is key 8 (r/4) + 4 hi + r%4
      if (r0 + kDecTile > c1) {
#pragma unroll
        for (int r = 0; r < 16; ++r)
          if (r0 + 8 * (r / 4) + 4 * hi + r % 4 >= c1) S[r] = -INFINITY;
      }
      float mx = fmaxf(S[0], S[1]);
#pragma unroll
      for (int r = 2; r < 16; r += 2) mx = fmaxf(fmaxf(mx, S[r]), S[r + 1]);
      mx = dec_half_max(mx);                      // finite: the tile has at least one row < c1
      const float m_new = fmaxf(m_run, mx);
      const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * c);  // 0 on the first tile
      const float mc = m_new * c;
      m_run = m_new;
      bf16x8 P[2];
      float ps = 0.f;
      const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
#pragma unroll
      for (int h2 = 0; h2 < 2; ++h2) {
        f32x8 e;
#pragma unroll
        for (int t = 0; t < 8; ++t) e[t] = __builtin_amdgcn_exp2f(fmaf(S[8 * h2 + t], c, -mc));
        const bf16x8 pb = __builtin_convertvector(e, bf16x8);
        P[h2] = pb;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          const bf16x2 pr = {pb[2 * t], pb[2 * t + 1]};
          ps = __builtin_amdgcn_fdot2_f32_bf16(pr, ones, ps, false);
        }
      }
      l_run = l_run * alpha + ps;
#pragma unroll
      for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int r = 0; r < 16; ++r) O[nb][r] *= alpha;
      // O^T += V^T P^T
#pragma unroll
      for (int h2 = 0; h2 < 2; ++h2)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
          const LDS_AS s16x4 *p0 = (const LDS_AS s16x4 *)(tile + voff[nb] + 16 * h2 * kRowBytes);
          const LDS_AS s16x4 *p1 = (const LDS_AS s16x4 *)(tile + voff[nb] + (16 * h2 + 8) * kRowBytes);
          const s16x4 v0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4 *)p0);
          const s16x4 v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_AS s16x4 *)p1);
          const bf16x8 va = __builtin_bit_cast(bf16x8, __builtin_shufflevector(v0, v1, 0, 1, 2, 3, 4, 5, 6, 7));
          O[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, P[h2], O[nb], 0, 0, 0);
        }
    }
    // the row sum of a head is split over the two half-waves (keys 4 hi + ...): add them up
    l_run = dec_half_sum(l_run);

    // ---- this window's partial: the four waves meet in LDS (over the tiles: everyone is done)
    __syncthreads();
    float *mg = (float *)&tiles[0][0];  // [wave][head][D + 2]: acc, then m, l
    if (col < live) {
      float *dst = mg + ((long long)wave * kDecHeads + col) * (D + 2);
#pragma unroll
      for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4)
#pragma unroll
          for (int x = 0; x < 4; ++x) dst[32 * nb + 8 * g4 + 4 * hi + x] = O[nb][4 * g4 + x];
      if (hi == 0) {
        dst[D] = m_run;
        dst[D + 1] = l_run;
      }
    }
    __syncthreads();
    for (int idx = tid; idx < live * (D / 4); idx += 256) {
      const int h = idx / (D / 4), d = (idx % (D / 4)) * 4;
      float mx = -INFINITY;
#pragma unroll
      for (int wv = 0; wv < 4; ++wv) mx = fmaxf(mx, mg[((long long)wv * kDecHeads + h) * (D + 2) + D]);
      float l = 0.f;
      f32x4 o = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int wv = 0; wv < 4; ++wv) {
        const float *src = mg + ((long long)wv * kDecHeads + h) * (D + 2);
        const float wgt = (src[D] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f((src[D] - mx) * c);
        l += src[D + 1] * wgt;
#pragma unroll
        for (int x = 0; x < 4; ++x) o[x] += src[d + x] * wgt;
      }
      float *slot = slots + (ws_slot_base(p, a.geom, b, head0 + h) + split) * ws_slot_floats(D);
      *(f32x4 *)(slot + d) = o;
      if (d == 0) *(float2 *)(slot + D) = float2{mx, l};
    }
    if (tid == 0 && c1 == hi_ && head_pass == 0) counts[w] = split + 1;
    __syncthreads();  // the merge area is tile space again
  }
}

int decode_mfma_resident(int D) {
  static ResidentCount count[2];
  return D == 128 ? count[1].get((const void *)decode_split_mfma_kernel<128>, 256, 0)
                  : count[0].get((const void *)decode_split_mfma_kernel<64>, 256, 0);
}

hipError_t launch_decode_split_mfma(const Problem &p, const DecodeArgs &a, long long blocks, hipStream_t st) {
  for (int pass = 0; pass < (p.g + kDecHeads - 1) / kDecHeads; ++pass) {
    if (p.D == 128)
      hipLaunchKernelGGL(decode_split_mfma_kernel<128>, dim3((unsigned)blocks), dim3(256), 0, st, p, a, pass);
    else
      hipLaunchKernelGGL(decode_split_mfma_kernel<64>, dim3((unsigned)blocks), dim3(256), 0, st, p, a, pass);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace segattn
