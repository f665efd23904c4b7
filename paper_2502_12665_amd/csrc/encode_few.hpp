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

// The same for one wave per (key, subspace) pair: a lane evaluates centroids lane, lane + 64, lane + 128
// and lane + 192 (keeping the nearest, the lower index on ties, in ascending order), then the wave picks
// the nearest of its lanes.  No barrier and no LDS, so the waves of a workgroup are independent: the
// decode prologues give their encoding workgroups sixteen pairs each instead of four.  Same arithmetic
// per centroid and the same tie rule as encode_few_pair, hence the same codes.
template <int DS>
__device__ __forceinline__ void encode_few_wave(const float* __restrict__ keys,
                                                const float* __restrict__ codebook,
                                                const float* __restrict__ weights, int mode,
                                                uint8_t* __restrict__ codes, int Hkv, int M, int n_new,
                                                int pos0, int64_t ctx_stride, long pair, int lane) {
  constexpr int D = 128, PER = kCentroids / 64;
  const int m = (int)(pair % M), j = (int)((pair / M) % n_new), bkv = (int)(pair / ((long)M * n_new));
  const int kv = bkv % Hkv, blk = kv * M + m;
  const float* kp = keys + ((size_t)bkv * n_new + j) * D + m * DS;
  float cw[PER][DS], kf[DS];
#pragma unroll
  for (int i = 0; i < PER; ++i)
#pragma unroll
    for (int t = 0; t < DS; ++t) cw[i][t] = codebook[((size_t)blk * kCentroids + lane + 64 * i) * DS + t];
#pragma unroll
  for (int t = 0; t < DS; ++t) kf[t] = kp[t];
  // (the weights are the same for every lane; they are read where they are used rather than kept in
  // DS * DS registers)
  const float* hd = weights ? weights + (size_t)kv * D + m * DS : nullptr;
  const float* H = weights ? weights + (size_t)blk * DS * DS : nullptr;
  double dist = 0.0;
  int idx = lane;
#pragma unroll
  for (int i = 0; i < PER; ++i) {
    double dv[DS], di = 0.0;
#pragma unroll
    for (int t = 0; t < DS; ++t) dv[t] = (double)kf[t] - (double)cw[i][t];
    if (mode == A2ATS_W_NONE) {
#pragma unroll
      for (int t = 0; t < DS; ++t) di += dv[t] * dv[t];
    } else if (mode == A2ATS_W_DIAG) {
#pragma unroll
      for (int t = 0; t < DS; ++t) di += dv[t] * (double)hd[t] * dv[t];
    } else {
#pragma unroll
      for (int r = 0; r < DS; ++r)
#pragma unroll
        for (int cc = 0; cc < DS; ++cc) di += dv[r] * (double)H[r * DS + cc] * dv[cc];
    }
    if (i == 0 || di < dist) {   // ascending index: a later equal distance does not replace
      dist = di;
      idx = lane + 64 * i;
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
  if (lane == 0) codes[((size_t)bkv * ctx_stride + pos0 + j) * M + m] = (uint8_t)idx;
}

// Pairs an encoding workgroup of a decode prologue takes: one per wave and sweep, `sweeps` of them, so
// that a launch has at most about 128 such workgroups beside those that build the tables (the
// prologue kernels hold one 1024-thread workgroup per CU: more would wait for a second round).
constexpr int kFewPairsPerSweep = 16;
inline int encode_few_sweeps(long n_pairs) {
  const long s = (n_pairs + 128L * kFewPairsPerSweep - 1) / (128L * kFewPairsPerSweep);
  return (int)(s < 1 ? 1 : s);
}

constexpr int kFewKeys = 32;   // at or below this many new keys per sequence the append-time kernel runs

}  // namespace a2ats
