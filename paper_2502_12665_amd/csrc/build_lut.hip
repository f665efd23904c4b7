// Steps 1-2 of a decode step: WRoPE query rotation (section 4.1: q~ = q R_b) and the
// per-subspace query x centroid tables (section 4.2 last equation, tabulated per subspace),
// written in the 32-bit fixed-point, head-interleaved layout the scoring kernels gather from.
//
// One workgroup per (sequence, KV head, group of 4 query heads).  The contraction is
// 2*B*Hq*256*D flop in total (8.4 Mflop at the 131072-token configuration), far below
// anything a matrix core would help with, so it runs on the vector ALU in float64: products
// of two float32 values are exact in float64, which makes every table entry the correctly
// rounded inner product.
#include "common.hpp"
#include "internal.hpp"

namespace a2ats {

constexpr int kLutThreads = 1024;

template <int DS, bool QBF16>
__global__ __launch_bounds__(kLutThreads) void build_lut_kernel(
    const void* __restrict__ q_in, const float* __restrict__ cos_b, const float* __restrict__ sin_b,
    const float* __restrict__ codebook, float* __restrict__ q_rot, int32_t* __restrict__ lut,
    float* __restrict__ lut_scale, int Hq, int Hkv, int NG) {
  constexpr int D = 128, HALF = 64, M = D / DS;
  constexpr int ENTRIES = kCentroids * M;
  constexpr int EPT = ENTRIES / kLutThreads;
  __shared__ float s_q[kHeadsPerGroup][D];
  __shared__ double s_max[kLutThreads / 64][kHeadsPerGroup];
  __shared__ int s_exp[kHeadsPerGroup];

  const int G = Hq / Hkv;
  const int g4 = blockIdx.x % NG;
  const int kv = (blockIdx.x / NG) % Hkv;
  const int b = blockIdx.x / (NG * Hkv);
  const int tid = threadIdx.x;

  // --- q~ = q R_b for the (up to) four heads of this group
  if (tid < kHeadsPerGroup * HALF) {
    const int r = tid / HALF, t = tid % HALF;
    const int hg = g4 * kHeadsPerGroup + r;
    float o1 = 0.f, o2 = 0.f;
    if (hg < G) {
      const int h = kv * G + hg;
      const size_t base = ((size_t)b * Hq + h) * D;
      double x1, x2;
      if (QBF16) {
        const uint16_t* qp = (const uint16_t*)q_in;
        x1 = (double)bf16_to_f32(qp[base + t]);
        x2 = (double)bf16_to_f32(qp[base + t + HALF]);
      } else {
        const float* qp = (const float*)q_in;
        x1 = (double)qp[base + t];
        x2 = (double)qp[base + t + HALF];
      }
      const double c = (double)cos_b[t], s = (double)sin_b[t];
      o1 = (float)(x1 * c - x2 * s);
      o2 = (float)(x2 * c + x1 * s);
      q_rot[base + t] = o1;
      q_rot[base + t + HALF] = o2;
    }
    s_q[r][t] = o1;
    s_q[r][t + HALF] = o2;
  }
  __syncthreads();

  // --- table entries in float64, in output order (c major, m minor)
  double val[EPT][kHeadsPerGroup];
  double mx[kHeadsPerGroup] = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
  for (int k = 0; k < EPT; ++k) {
    const int e = tid + k * kLutThreads;
    const int c = e / M, m = e % M;
    const float* cw = codebook + (((size_t)kv * M + m) * kCentroids + c) * DS;
    float cv[DS];
#pragma unroll
    for (int t = 0; t < DS; t += 4) {
      const float4 f = *(const float4*)(cw + t);
      cv[t] = f.x; cv[t + 1] = f.y; cv[t + 2] = f.z; cv[t + 3] = f.w;
    }
#pragma unroll
    for (int r = 0; r < kHeadsPerGroup; ++r) {
      double acc = 0.0;
#pragma unroll
      for (int t = 0; t < DS; ++t) acc += (double)s_q[r][m * DS + t] * (double)cv[t];
      val[k][r] = acc;
      mx[r] = fmax(mx[r], fabs(acc));
    }
  }

  // --- per-head power-of-two scale: M * max|entry| * 2^e < 2^30
#pragma unroll
  for (int r = 0; r < kHeadsPerGroup; ++r) {
    double v = mx[r];
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v = fmax(v, __shfl_xor(v, off));
    if ((tid & 63) == 0) s_max[tid >> 6][r] = v;
  }
  __syncthreads();
  if (tid < kHeadsPerGroup) {
    double v = 0.0;
    for (int w = 0; w < kLutThreads / 64; ++w) v = fmax(v, s_max[w][tid]);
    int e = 0;
    if (v > 0.0) {
      int x;
      frexp(v * (double)M, &x);   // v*M < 2^x
      e = 30 - x;
      e = e > 100 ? 100 : (e < -100 ? -100 : e);
    }
    s_exp[tid] = e;
    const int hg = g4 * kHeadsPerGroup + tid;
    if (hg < G) lut_scale[(size_t)b * Hq + kv * G + hg] = (float)ldexp(1.0, -e);
  }
  __syncthreads();

  int4* out = (int4*)(lut + (size_t)blockIdx.x * ENTRIES * kHeadsPerGroup);
  const int e0 = s_exp[0], e1 = s_exp[1], e2 = s_exp[2], e3 = s_exp[3];
#pragma unroll
  for (int k = 0; k < EPT; ++k) {
    int4 o;
    o.x = (int)rint(ldexp(val[k][0], e0));
    o.y = (int)rint(ldexp(val[k][1], e1));
    o.z = (int)rint(ldexp(val[k][2], e2));
    o.w = (int)rint(ldexp(val[k][3], e3));
    out[tid + k * kLutThreads] = o;
  }
}

hipError_t launch_build_lut(const a2ats_dims& d, const void* q, int q_dtype, const float* cos_b,
                            const float* sin_b, const float* codebook, float* q_rot, int32_t* lut,
                            float* lut_scale, hipStream_t stream) {
  const int G = d.n_q_heads / d.n_kv_heads;
  const int NG = (G + kHeadsPerGroup - 1) / kHeadsPerGroup;
  const dim3 grid(d.batch * d.n_kv_heads * NG), block(kLutThreads);
  if (grid.x == 0) return hipSuccess;
#define A2ATS_LAUNCH_LUT(DS, BF)                                                            \
  hipLaunchKernelGGL((build_lut_kernel<DS, BF>), grid, block, 0, stream, q, cos_b, sin_b,    \
                     codebook, q_rot, lut, lut_scale, d.n_q_heads, d.n_kv_heads, NG)
  if (d.sub_dim == 8) {
    if (q_dtype == A2ATS_BF16) A2ATS_LAUNCH_LUT(8, true); else A2ATS_LAUNCH_LUT(8, false);
  } else {
    if (q_dtype == A2ATS_BF16) A2ATS_LAUNCH_LUT(4, true); else A2ATS_LAUNCH_LUT(4, false);
  }
#undef A2ATS_LAUNCH_LUT
  return hipGetLastError();
}

}  // namespace a2ats
