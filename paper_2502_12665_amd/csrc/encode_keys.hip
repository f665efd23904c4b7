// Prefill / append-side key encoder: query-aware quantisation function f' of section 4.2
// (f of section 2.2 when H = I), per subspace:
//     code = argmin_c (k_m - C[m,c]) H_m (k_m - C[m,c])^T ,  lowest c on exact ties.
//
// The work is 256 small distance evaluations per subvector: plain float32 vector ALU work
// (about 100 kflop per key, 200 flop per byte read), not a matrix-core shape -- the inner
// dimension is ds = 4 or 8 and the expanded ||c||^2 - 2 k.c form would lose the bits the
// argmin is decided by.  Following the Cholesky reformulation of section 4.2 (H = L L^T,
// z = k L, c^z = c L), keys and centroids are first mapped to the space where the distortion
// is the plain squared distance, so the inner loop is `sub, fma` per dimension whatever the
// weighting; sqrt(h) takes the place of L for per-dimension weights.  One thread owns one
// key subvector; the centroid stream is wave-uniform and comes through the scalar data path.
// Whenever the two smallest float32 distances are within rounding reach of each other the
// thread re-evaluates all 256 distortions in float64 straight from the definition, so the
// emitted code is the float64 argmin.
#include "common.hpp"
#include "internal.hpp"
#include "encode_few.hpp"

namespace a2ats {

constexpr int kEncThreads = 256;

size_t encode_ws_bytes(const a2ats_dims& d) {
  const size_t blocks = (size_t)d.n_kv_heads * d.n_sub;
  return blocks * d.sub_dim * d.sub_dim * sizeof(float) +
         blocks * kCentroids * d.sub_dim * sizeof(float);
}

// One workgroup per (KV head, subspace): transform matrix T (z = k T) and transformed centroids.
template <int DS>
__global__ __launch_bounds__(kCentroids) void encode_prepare_kernel(
    const float* __restrict__ codebook, const float* __restrict__ weights, int mode, int M,
    float* __restrict__ tmat, float* __restrict__ cz) {
  __shared__ double s_T[DS][DS];
  const int blk = blockIdx.x;          // kv * M + m
  const int kv = blk / M, m = blk % M;
  if (threadIdx.x == 0) {
    for (int r = 0; r < DS; ++r)
      for (int c = 0; c < DS; ++c) s_T[r][c] = 0.0;
    if (mode == A2ATS_W_DIAG) {
      for (int t = 0; t < DS; ++t) s_T[t][t] = sqrt((double)weights[(size_t)kv * M * DS + m * DS + t]);
    } else {   // lower Cholesky factor of the ds x ds block
      const float* H = weights + (size_t)blk * DS * DS;
      for (int r = 0; r < DS; ++r)
        for (int c = 0; c <= r; ++c) {
          double s = (double)H[r * DS + c];
          for (int t = 0; t < c; ++t) s -= s_T[r][t] * s_T[c][t];
          s_T[r][c] = (r == c) ? sqrt(s > 0.0 ? s : 0.0) : (s_T[c][c] > 0.0 ? s / s_T[c][c] : 0.0);
        }
    }
    for (int r = 0; r < DS; ++r)
      for (int c = 0; c < DS; ++c) tmat[(size_t)blk * DS * DS + r * DS + c] = (float)s_T[r][c];
  }
  __syncthreads();
  const int c = threadIdx.x;
  const float* cw = codebook + ((size_t)blk * kCentroids + c) * DS;
#pragma unroll
  for (int t = 0; t < DS; ++t) {
    double s = 0.0;
#pragma unroll
    for (int r = 0; r < DS; ++r) s += (double)cw[r] * s_T[r][t];
    cz[((size_t)blk * kCentroids + c) * DS + t] = (float)s;
  }
}

template <int DS, int MODE>
__global__ __launch_bounds__(kEncThreads) void encode_kernel(
    const float* __restrict__ keys, const float* __restrict__ codebook,
    const float* __restrict__ weights, const float* __restrict__ tmat, const float* __restrict__ cz,
    uint8_t* __restrict__ codes, int Hkv, int M, int n_new, int pos0, int64_t ctx_stride) {
  constexpr int D = 128;
  const int m = blockIdx.x;
  const int j = blockIdx.y * kEncThreads + threadIdx.x;
  const int bkv = blockIdx.z, kv = bkv % Hkv;
  if (j >= n_new) return;
  const int blk = kv * M + m;

  float ks[DS];
  {
    const float* kp = keys + ((size_t)bkv * n_new + j) * D + m * DS;
#pragma unroll
    for (int t = 0; t < DS; t += 4) {
      const float4 f = *(const float4*)(kp + t);
      ks[t] = f.x; ks[t + 1] = f.y; ks[t + 2] = f.z; ks[t + 3] = f.w;
    }
  }
  float z[DS];
  const float* cp;
  if (MODE == A2ATS_W_NONE) {
#pragma unroll
    for (int t = 0; t < DS; ++t) z[t] = ks[t];
    cp = codebook + (size_t)blk * kCentroids * DS;
  } else {
    const float* T = tmat + (size_t)blk * DS * DS;
#pragma unroll
    for (int t = 0; t < DS; ++t) {
      float s = 0.f;
#pragma unroll
      for (int r = 0; r < DS; ++r) s += ks[r] * T[r * DS + t];
      z[t] = s;
    }
    cp = cz + (size_t)blk * kCentroids * DS;
  }
  float zz = 0.f;
#pragma unroll
  for (int t = 0; t < DS; ++t) zz += z[t] * z[t];

  // The centroid index rides in the low 8 mantissa bits of the distance.  Distances are >= 0, so
  // their bit patterns order like the values and the tracking is done on unsigned integers
  // (no denormal or NaN handling in the way): one minimum tracks the smallest distance together
  // with its index, the lower index winning among distances equal in the remaining 16 mantissa
  // bits; anything that close is re-decided in float64 below.
  uint32_t k1 = 0x7f800000u, k2 = 0x7f800000u;   // +inf
  const uint32_t keep = 0xffffff00u;
#pragma unroll 4
  for (int c = 0; c < kCentroids; ++c) {
    float d = 0.f;
#pragma unroll
    for (int t = 0; t < DS; ++t) {
      const float e = z[t] - cp[c * DS + t];
      d += e * e;
    }
    const uint32_t key = (__float_as_uint(d) & keep) | (uint32_t)c;
    asm("v_med3_u32 %0, %1, %2, %3" : "=v"(k2) : "v"(k1), "v"(k2), "v"(key));   // with k1 <= k2: the new second smallest
    k1 = min(k1, key);
  }
  int arg = (int)(k1 & 0xffu);
  const float b1 = __uint_as_float(k1 & keep), b2 = __uint_as_float(k2 & keep);

  // float32 rounding reach of a distance: a few ulp of (|z| + |c|)^2-sized terms
  const float tol = 1e-4f * b2 + 4e-6f * zz + 1e-30f;
  if (!(b2 - b1 > tol)) {
    const float* cw0 = codebook + (size_t)blk * kCentroids * DS;
    double best = INFINITY;
    int a64 = 0;
    for (int c = 0; c < kCentroids; ++c) {
      double dv[DS];
#pragma unroll
      for (int t = 0; t < DS; ++t) dv[t] = (double)ks[t] - (double)cw0[c * DS + t];
      double dist = 0.0;
      if (MODE == A2ATS_W_NONE) {
#pragma unroll
        for (int t = 0; t < DS; ++t) dist += dv[t] * dv[t];
      } else if (MODE == A2ATS_W_DIAG) {
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
      if (dist < best) {
        best = dist;
        a64 = c;
      }
    }
    arg = a64;
  }
  codes[((size_t)bkv * ctx_stride + pos0 + j) * M + m] = (uint8_t)arg;
}

// Append-time shape (a few new keys per sequence, e.g. one per decode step): the prefill kernel
// would run one thread per key with 256 serial distance evaluations; here a workgroup of 256
// threads takes one (key, subspace) pair (see encode_few.hpp).
template <int DS>
__global__ __launch_bounds__(kCentroids) void encode_few_kernel(
    const float* __restrict__ keys, const float* __restrict__ codebook,
    const float* __restrict__ weights, int mode, uint8_t* __restrict__ codes, int Hkv, int M,
    int n_new, int pos0, int64_t ctx_stride) {
  __shared__ double s_d[4];
  __shared__ int s_i[4];
  encode_few_pair<DS>(keys, codebook, weights, mode, codes, Hkv, M, n_new, pos0, ctx_stride, blockIdx.x,
                      blockIdx.y, blockIdx.z, threadIdx.x, 0, true, s_d, s_i);
}

template <int DS>
static hipError_t launch_encode_ds(const a2ats_dims& d, const float* keys, int n_new, int pos0,
                                   const float* codebook, const float* weights, int mode, uint8_t* codes,
                                   void* ws, hipStream_t stream) {
  const int M = d.n_sub, Hkv = d.n_kv_heads;
  if (n_new <= kFewKeys) {
    hipLaunchKernelGGL((encode_few_kernel<DS>), dim3(M, n_new, d.batch * Hkv), dim3(kCentroids), 0, stream,
                       keys, codebook, weights, mode, codes, Hkv, M, n_new, pos0, d.ctx_stride);
    return hipGetLastError();
  }
  float* tmat = (float*)ws;
  float* cz = tmat ? tmat + (size_t)Hkv * M * DS * DS : nullptr;
  if (mode != A2ATS_W_NONE) {
    hipLaunchKernelGGL((encode_prepare_kernel<DS>), dim3(Hkv * M), dim3(kCentroids), 0, stream, codebook,
                       weights, mode, M, tmat, cz);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
  }
  const dim3 grid(M, (n_new + kEncThreads - 1) / kEncThreads, d.batch * Hkv), block(kEncThreads);
#define A2ATS_LAUNCH_ENC(MODE)                                                                      \
  hipLaunchKernelGGL((encode_kernel<DS, MODE>), grid, block, 0, stream, keys, codebook, weights, tmat, \
                     cz, codes, Hkv, M, n_new, pos0, d.ctx_stride)
  if (mode == A2ATS_W_NONE) A2ATS_LAUNCH_ENC(A2ATS_W_NONE);
  else if (mode == A2ATS_W_DIAG) A2ATS_LAUNCH_ENC(A2ATS_W_DIAG);
  else A2ATS_LAUNCH_ENC(A2ATS_W_BLOCK);
#undef A2ATS_LAUNCH_ENC
  return hipGetLastError();
}

hipError_t launch_encode(const a2ats_dims& d, const float* keys, int n_new, int pos0, const float* codebook,
                         const float* weights, int mode, uint8_t* codes, void* ws, hipStream_t stream) {
  if (n_new == 0 || d.batch == 0) return hipSuccess;
  if (d.sub_dim == 8)
    return launch_encode_ds<8>(d, keys, n_new, pos0, codebook, weights, mode, codes, ws, stream);
  return launch_encode_ds<4>(d, keys, n_new, pos0, codebook, weights, mode, codes, ws, stream);
}

}  // namespace a2ats
