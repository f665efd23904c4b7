// Offline codebook construction (section 4.2): the second moment of the rotated queries,
//     H = E[q~^T q~]   (one D x D matrix per KV head; the G query heads of a KV head are pooled),
// and the centroid step of k-means under the query-aware distortion.  The paper runs k-means on
// z = k L and maps the centroids back with L^-1; the mean is linear, so the new codeword is the
// mean of the keys assigned to it, and a Lloyd iteration is a2ats_encode_keys (assignment under
// (k - c) H (k - c)^T) followed by a2ats_codebook_update.  Both geometries: codewords are
// [Hkv][M][L][ds], and a key contributes its subvector m to codeword codes[j][m] of subspace m.
//
//   second_moment_kernel     a workgroup accumulates the 128 x 128 outer-product sum of its share of
//                            the samples in float64 (an 8 x 8 block per thread), one partial each
//   second_moment_sum_kernel adds the partials in a fixed order, divides, rounds once to float32
//   update_clear_kernel      zeroes the float64 sums and the counts
//   update_add_kernel        one thread per (key, dimension): hardware float64 atomic adds into the
//                            sums (the order of the additions, and so the last bits, vary from run
//                            to run), one count per (key, subspace)
//   update_mean_kernel       sum / count, rounded once; codewords without keys keep their value
#include "common.hpp"
#include "internal.hpp"

namespace a2ats {
namespace {

constexpr int kFD = 128;
constexpr int kMomentParts = 64;   // partial sums per KV head
constexpr int kMomentRows = 32;    // sample rows staged per step

__global__ __launch_bounds__(256) void second_moment_kernel(const float* __restrict__ q_rot, double* __restrict__ part,
                                                            int Hq, int Hkv, long rows) {
  // rows = n_samples * G row vectors of this KV head: row r is sample r / G, head kv * G + r % G
  __shared__ float s_x[kMomentRows][kFD];
  const int kv = blockIdx.y, p = blockIdx.x, tid = threadIdx.x, G = Hq / Hkv;
  const int ti = (tid >> 4) * 8, tj = (tid & 15) * 8;   // this thread's 8 x 8 block of H
  double acc[8][8];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[i][j] = 0.0;
  for (long r0 = (long)p * kMomentRows; r0 < rows; r0 += (long)kMomentParts * kMomentRows) {
    __syncthreads();
    for (int e = tid; e < kMomentRows * (kFD / 4); e += 256) {
      const int rr = e / (kFD / 4), c4 = e % (kFD / 4);
      const long r = r0 + rr;
      float4 f = make_float4(0.f, 0.f, 0.f, 0.f);   // rows past the end add nothing
      if (r < rows) f = *(const float4*)(q_rot + ((size_t)(r / G) * Hq + kv * G + r % G) * kFD + 4 * c4);
      *(float4*)&s_x[rr][4 * c4] = f;
    }
    __syncthreads();
    for (int rr = 0; rr < kMomentRows; ++rr) {
      double a[8], b[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) a[i] = (double)s_x[rr][ti + i], b[i] = (double)s_x[rr][tj + i];
#pragma unroll
      for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[i][j] += a[i] * b[j];
    }
  }
  double* out = part + ((size_t)kv * kMomentParts + p) * kFD * kFD;
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int j = 0; j < 8; ++j) out[(ti + i) * kFD + tj + j] = acc[i][j];
}

__global__ __launch_bounds__(256) void second_moment_sum_kernel(const double* __restrict__ part, float* __restrict__ h,
                                                                double inv_rows) {
  const int kv = blockIdx.y, e = blockIdx.x * 256 + threadIdx.x;   // e < 128 * 128
  double s = 0.0;
  for (int p = 0; p < kMomentParts; ++p) s += part[((size_t)kv * kMomentParts + p) * kFD * kFD + e];
  h[(size_t)kv * kFD * kFD + e] = (float)(s * inv_rows);
}

__global__ void update_clear_kernel(double* __restrict__ sums, uint32_t* __restrict__ counts, size_t n_sums,
                                    size_t n_counts) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_sums; i += (size_t)gridDim.x * blockDim.x)
    sums[i] = 0.0;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_counts; i += (size_t)gridDim.x * blockDim.x)
    counts[i] = 0u;
}

template <typename CODE>
__global__ __launch_bounds__(256) void update_add_kernel(const float* __restrict__ keys, const CODE* __restrict__ codes,
                                                         double* __restrict__ sums, uint32_t* __restrict__ counts,
                                                         int Hkv, int M, int L, int ds, int n_new, int pos0,
                                                         int64_t ctx_stride) {
  const int bkv = blockIdx.y, kv = bkv % Hkv, tid = threadIdx.x;
  const long j = (long)blockIdx.x * 2 + (tid >> 7);   // two keys per workgroup
  const int t = tid & 127;
  if (j >= n_new) return;
  const int m = t / ds;
  const int c = (int)codes[((size_t)bkv * ctx_stride + pos0 + j) * M + m] & (L - 1);   // L is a power of two
  const size_t cw = ((size_t)kv * M + m) * L + c;
  unsafeAtomicAdd(&sums[cw * ds + t % ds], (double)keys[((size_t)bkv * n_new + j) * kFD + t]);
  if (t % ds == 0) atomicAdd(&counts[cw], 1u);
}

__global__ __launch_bounds__(256) void update_mean_kernel(const double* __restrict__ sums,
                                                          const uint32_t* __restrict__ counts,
                                                          const float* __restrict__ old_cb, float* __restrict__ new_cb,
                                                          int32_t* __restrict__ counts_out, int ds, size_t n_elems) {
  const size_t e = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (e >= n_elems) return;
  const size_t cw = e / ds;
  const uint32_t n = counts[cw];
  new_cb[e] = n ? (float)(sums[e] / (double)n) : old_cb[e];
  if (counts_out && e % ds == 0) counts_out[cw] = (int32_t)n;
}

}  // namespace

size_t fit_ws_bytes(const a2ats_dims& d) {
  const size_t moment = (size_t)d.n_kv_heads * kMomentParts * kFD * kFD * sizeof(double);
  const size_t cws = (size_t)d.n_kv_heads * d.n_sub * d.n_centroids;
  const size_t update = cws * d.sub_dim * sizeof(double) + cws * sizeof(uint32_t);
  return ((moment > update ? moment : update) + 255) & ~(size_t)255;
}

hipError_t launch_second_moment(const a2ats_dims& d, const float* q_rot, int64_t n_samples, float* h_out, void* ws,
                                hipStream_t stream) {
  if (d.n_kv_heads == 0) return hipSuccess;
  const int G = d.n_q_heads / d.n_kv_heads;
  const long rows = (long)n_samples * G;
  hipLaunchKernelGGL(second_moment_kernel, dim3(kMomentParts, d.n_kv_heads), dim3(256), 0, stream, q_rot, (double*)ws,
                     d.n_q_heads, d.n_kv_heads, rows);
  hipError_t err = hipGetLastError();
  if (err != hipSuccess) return err;
  hipLaunchKernelGGL(second_moment_sum_kernel, dim3(kFD * kFD / 256, d.n_kv_heads), dim3(256), 0, stream,
                     (const double*)ws, h_out, rows > 0 ? 1.0 / (double)rows : 0.0);
  return hipGetLastError();
}

hipError_t launch_codebook_update(const a2ats_dims& d, const float* keys, int n_new, int pos0, const void* codes,
                                  const float* codebook, float* codebook_out, int32_t* counts_out, void* ws,
                                  hipStream_t stream) {
  const size_t cws = (size_t)d.n_kv_heads * d.n_sub * d.n_centroids, n_elems = cws * d.sub_dim;
  if (n_elems == 0) return hipSuccess;
  double* sums = (double*)ws;
  uint32_t* counts = (uint32_t*)(sums + n_elems);
  hipLaunchKernelGGL(update_clear_kernel, dim3(1024), dim3(256), 0, stream, sums, counts, n_elems, cws);
  hipError_t err = hipGetLastError();
  if (err != hipSuccess) return err;
  if (n_new > 0 && d.batch > 0) {
    const dim3 grid((n_new + 1) / 2, d.batch * d.n_kv_heads);
    if (single_codebook(d))
      hipLaunchKernelGGL(update_add_kernel<uint16_t>, grid, dim3(256), 0, stream, keys, (const uint16_t*)codes, sums,
                         counts, d.n_kv_heads, d.n_sub, d.n_centroids, d.sub_dim, n_new, pos0, d.ctx_stride);
    else
      hipLaunchKernelGGL(update_add_kernel<uint8_t>, grid, dim3(256), 0, stream, keys, (const uint8_t*)codes, sums,
                         counts, d.n_kv_heads, d.n_sub, d.n_centroids, d.sub_dim, n_new, pos0, d.ctx_stride);
    if ((err = hipGetLastError()) != hipSuccess) return err;
  }
  hipLaunchKernelGGL(update_mean_kernel, dim3((unsigned)((n_elems + 255) / 256)), dim3(256), 0, stream, sums, counts,
                     codebook, codebook_out, counts_out, d.sub_dim, n_elems);
  return hipGetLastError();
}

}  // namespace a2ats
