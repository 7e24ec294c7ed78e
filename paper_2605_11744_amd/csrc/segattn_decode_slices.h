// Slice search shared by the two decode split kernels of libsegattn.
#pragma once
#include "segattn_internal.h"

namespace segattn {

// The windows of all (sequence, KV head) pairs laid end to end in the order b * Hkv + kv; workgroup
// i owns rows [i * rows_per_wg, (i + 1) * rows_per_wg) of that sequence.  Finds the window that holds
// the workgroup's first row and the row's offset inside it: every thread adds up a run of windows,
// thread 0 walks the 256 run sums and then the run.  w = -1 if the slices before this one cover
// every row.  Called by all 256 threads of the workgroup (it synchronises).
__device__ inline void decode_window_rows(const Problem &p, const DecodeArgs &a, int w, int &lo, int &hi) {
  const int kv = w % p.Hkv;
  const int *meta = meta_ro(a.cache, a.geom, p, w / p.Hkv, kv);
  int seg_row0;
  window_of(p, a.geom, kv, meta, lo, seg_row0);
  hi = seg_row0 + meta[META_FILL];
}

__device__ inline void decode_slice_start(const Problem &p, const DecodeArgs &a, long long start, int &w_out,
                                          int &off_out) {
  __shared__ long long sm_run[256];
  __shared__ int sm_start[2];
  const int tid = threadIdx.x;
  const int n_win = p.B * p.Hkv;
  const int run = (n_win + 255) / 256;
  {
    long long sum = 0;
    for (int j = 0; j < run; ++j) {
      const int w = tid * run + j;
      if (w < n_win) {
        int lo, hi;
        decode_window_rows(p, a, w, lo, hi);
        sum += hi - lo;
      }
    }
    sm_run[tid] = sum;
  }
  __syncthreads();
  if (tid == 0) {
    long long before = 0;
    int t = 0;
    while (t < 256 && before + sm_run[t] <= start) before += sm_run[t++];
    int w = t * run, found = -1;
    for (int j = 0; t < 256 && j < run && w < n_win; ++j, ++w) {
      int lo, hi;
      decode_window_rows(p, a, w, lo, hi);
      if (before + (hi - lo) > start) {
        found = w;
        break;
      }
      before += hi - lo;
    }
    sm_start[0] = found;
    sm_start[1] = (int)(start - before);
  }
  __syncthreads();
  w_out = __builtin_amdgcn_readfirstlane(sm_start[0]);
  off_out = __builtin_amdgcn_readfirstlane(sm_start[1]);
}

}  // namespace segattn
