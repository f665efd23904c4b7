// Append-time key encoding (section 4.2: argmin_c (k - c) H (k - c)^T per subspace) for a few new
// keys: a group of 256 threads takes one (key, subspace) pair, one thread per centroid evaluates
// the distortion straight from the definition in float64, and an argmin over the group picks the
// winner, lowest index on ties.  Shared by the stand-alone encoder and the fused decode prologue.
#pragma once

#include "common.hpp"

namespace a2ats {

// Called by every thread of the workgroup (it contains a barrier); `c` is the thread's index in
// its 256-thread group, `grp` the group's index in the workgroup, `active` whether the group has
// a pair to encode.  s_d / s_i: 4 entries of LDS per group.
template <int DS>
__device__ __forceinline__ void encode_few_pair(const float* __restrict__ keys,
                                                const float* __restrict__ codebook,
                                                const float* __restrict__ weights, int mode,
                                                uint8_t* __restrict__ codes, int Hkv, int M, int n_new,
                                                int pos0, int64_t ctx_stride, int m, int j, int bkv, int c,
                                                int grp, bool active, double* s_d, int* s_i) {
  constexpr int D = 128;
  double dist = 0.0;
  int idx = c;
  if (active) {
    const int kv = bkv % Hkv, blk = kv * M + m;
    const float* kp = keys + ((size_t)bkv * n_new + j) * D + m * DS;
    const float* cw = codebook + ((size_t)blk * kCentroids + c) * DS;
    double dv[DS];
#pragma unroll
    for (int t = 0; t < DS; ++t) dv[t] = (double)kp[t] - (double)cw[t];
    if (mode == A2ATS_W_NONE) {
#pragma unroll
      for (int t = 0; t < DS; ++t) dist += dv[t] * dv[t];
    } else if (mode == A2ATS_W_DIAG) {
      const float* hw = weights + (size_t)kv * D + m * DS;
#pragma unroll
      for (int t = 0; t < DS; ++t) dist += dv[t] * (double)hw[t] * dv[t];
    } else {
      const float* H = weights + (size_t)blk * DS * DS;
#pragma unroll
      for (int r = 0; r < DS; ++r)
#pragma unroll
        for (int cc = 0; cc < DS; ++cc) dist += dv[r] * (double)H[r * DS + cc] * dv[cc];
    }
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    const double od = __shfl_xor(dist, off);
    const int oi = __shfl_xor(idx, off);
    if (od < dist || (od == dist && oi < idx)) {
      dist = od;
      idx = oi;
    }
  }
  if ((c & 63) == 0) {
    s_d[grp * 4 + (c >> 6)] = dist;
    s_i[grp * 4 + (c >> 6)] = idx;
  }
  __syncthreads();
  if (active && c == 0) {
    for (int w = 1; w < kCentroids / 64; ++w)
      if (s_d[grp * 4 + w] < dist || (s_d[grp * 4 + w] == dist && s_i[grp * 4 + w] < idx)) {
        dist = s_d[grp * 4 + w];
        idx = s_i[grp * 4 + w];
      }
    codes[((size_t)bkv * ctx_stride + pos0 + j) * M + m] = (uint8_t)idx;
  }
}

constexpr int kFewKeys = 32;   // at or below this many new keys per sequence the append-time kernel runs

}  // namespace a2ats
