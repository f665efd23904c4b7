// Steps 1-2 of a decode step: WRoPE query rotation (section 4.1: q~ = q R_b) and the
// per-subspace query x centroid tables (section 4.2 last equation, tabulated per subspace).
//
// One workgroup per (sequence, KV head, group of 4 query heads).  The contraction is
// 2*B*Hq*256*D flop in total (8.4 Mflop at the 131072-token configuration), far below
// anything a matrix core would help with, so it runs on the vector ALU in float64: products
// of two float32 values are exact in float64, which makes every table entry the correctly
// rounded inner product.  Three things are written per head (see "Lookup-table format" in
// a2ats.h): the exact 32-bit fixed-point table [m][c], a 16-bit coarse copy of it interleaved
// over the four heads of the group [c][m][4] for the streaming kernel, and the two numbers that
// relate them (sum of the per-subspace minima, shift).
#include "common.hpp"
#include "internal.hpp"

namespace a2ats {

constexpr int kLutThreads = 1024;
constexpr int kLutWaves = kLutThreads / 64;

template <int DS, bool QBF16>
__global__ __launch_bounds__(kLutThreads) void build_lut_kernel(
    const void* __restrict__ q_in, const float* __restrict__ cos_b, const float* __restrict__ sin_b,
    const float* __restrict__ codebook, float* __restrict__ q_rot, int32_t* __restrict__ lut,
    float* __restrict__ lut_scale, int B, int Hq, int Hkv, int NG) {
  constexpr int D = 128, HALF = 64, M = D / DS;
  constexpr int ENTRIES = kCentroids * M;
  constexpr int EPT = ENTRIES / kLutThreads;
  constexpr int ROW = kCentroids + 1;   // padded row of the LDS transpose buffer
  constexpr int MAXQ = 65535 / M;       // a sum of M coarse entries fits 16 bits
  extern __shared__ __align__(16) unsigned char dyn_lds[];
  int32_t* s_t = (int32_t*)dyn_lds;     // [4][M][ROW]
  __shared__ float s_q[kHeadsPerGroup][D];
  __shared__ double s_max[kLutWaves][kHeadsPerGroup];
  __shared__ int s_exp[kHeadsPerGroup];
  __shared__ int32_t s_mm[kLutWaves][M][8];
  __shared__ int32_t s_min[M][kHeadsPerGroup];
  __shared__ int32_t s_shift[kHeadsPerGroup];

  const int G = Hq / Hkv;
  const int prob = blockIdx.x;
  const int g4 = prob % NG, kv = (prob / NG) % Hkv, b = prob / (NG * Hkv);
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const LutLayout lay = lut_layout(B, Hq, Hkv, M);

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

  // --- table entries in float64; entry e = c * M + m, so a thread's entries share m = tid % M
  double val[EPT][kHeadsPerGroup];
  double mx[kHeadsPerGroup] = {0.0, 0.0, 0.0, 0.0};
  const int m = tid % M;
#pragma unroll
  for (int k = 0; k < EPT; ++k) {
    const int c = (tid + k * kLutThreads) / M;
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
    if (lane == 0) s_max[wv][r] = v;
  }
  __syncthreads();
  if (tid < kHeadsPerGroup) {
    double v = 0.0;
    for (int w = 0; w < kLutWaves; ++w) v = fmax(v, s_max[w][tid]);
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

  // --- exact fixed-point entries; per-(subspace, head) minimum and maximum over the centroids
  int32_t iv[EPT][kHeadsPerGroup];
  int32_t mn[4] = {INT32_MAX, INT32_MAX, INT32_MAX, INT32_MAX};
  int32_t mxv[4] = {INT32_MIN, INT32_MIN, INT32_MIN, INT32_MIN};
#pragma unroll
  for (int k = 0; k < EPT; ++k)
#pragma unroll
    for (int r = 0; r < kHeadsPerGroup; ++r) {
      const int32_t v = (int32_t)rint(ldexp(val[k][r], s_exp[r]));
      iv[k][r] = v;
      mn[r] = min(mn[r], v);
      mxv[r] = max(mxv[r], v);
    }
#pragma unroll
  for (int off = M; off < 64; off <<= 1)
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      mn[r] = min(mn[r], __shfl_xor(mn[r], off));
      mxv[r] = max(mxv[r], __shfl_xor(mxv[r], off));
    }
  if (lane < M)
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      s_mm[wv][lane][r] = mn[r];
      s_mm[wv][lane][4 + r] = mxv[r];
    }
  __syncthreads();
  if (tid < M * 4) {   // thread (mm, r): min over waves, and the range max - min of this subspace
    const int mm = tid / 4, r = tid % 4;
    int32_t lo = s_mm[0][mm][r], hi = s_mm[0][mm][4 + r];
    for (int w = 1; w < kLutWaves; ++w) {
      lo = min(lo, s_mm[w][mm][r]);
      hi = max(hi, s_mm[w][mm][4 + r]);
    }
    s_min[mm][r] = lo;
    s_mm[0][mm][4 + r] = hi;   // only this thread reads or writes this slot from here on
  }
  __syncthreads();
  if (tid < kHeadsPerGroup) {
    const int r = tid;
    uint32_t range = 0;
    int32_t base = 0, top = 0;
    for (int mm = 0; mm < M; ++mm) {
      range = max(range, (uint32_t)(s_mm[0][mm][4 + r] - s_min[mm][r]));
      base += s_min[mm][r];
      top += s_mm[0][mm][4 + r];
    }
    int sh = 0;
    while ((range >> sh) > (uint32_t)MAXQ) ++sh;
    s_shift[r] = sh;
    const int hg = g4 * kHeadsPerGroup + r;
    if (hg < G) {
      int32_t* meta = lut + lay.off_meta + ((size_t)b * Hq + kv * G + hg) * 4;
      meta[0] = base;   // sum over subspaces of the smallest entry
      meta[1] = sh;     // coarse entry = (exact entry - subspace minimum) >> sh
      meta[2] = top;    // sum over subspaces of the largest entry: no score exceeds it
      meta[3] = 0;
    }
  }
  __syncthreads();

  // --- coarse table, [half][c][m & 15][4 heads] 16-bit: one 8-byte entry per (c, m)
  {
    uint2* coarse = (uint2*)(lut + lay.off_coarse) + (size_t)prob * ENTRIES;
    const int sh0 = s_shift[0], sh1 = s_shift[1], sh2 = s_shift[2], sh3 = s_shift[3];
    const int mn0 = s_min[m][0], mn1 = s_min[m][1], mn2 = s_min[m][2], mn3 = s_min[m][3];
#pragma unroll
    for (int k = 0; k < EPT; ++k) {
      const int c = (tid + k * kLutThreads) / M;
      const uint32_t q0 = (uint32_t)(iv[k][0] - mn0) >> sh0, q1 = (uint32_t)(iv[k][1] - mn1) >> sh1;
      const uint32_t q2 = (uint32_t)(iv[k][2] - mn2) >> sh2, q3 = (uint32_t)(iv[k][3] - mn3) >> sh3;
      coarse[(m >> 4) * (kCentroids * 16) + c * 16 + (m & 15)] = make_uint2(q0 | (q1 << 16), q2 | (q3 << 16));
    }
  }

  // --- exact tables, one per head as [m][c]: transposed through LDS so the writes are coalesced
#pragma unroll
  for (int k = 0; k < EPT; ++k) {
    const int c = (tid + k * kLutThreads) / M;
#pragma unroll
    for (int r = 0; r < kHeadsPerGroup; ++r) s_t[(r * M + m) * ROW + c] = iv[k][r];
  }
  __syncthreads();
  for (int i = tid; i < kHeadsPerGroup * ENTRIES; i += kLutThreads) {
    const int r = i / ENTRIES, mc = i % ENTRIES;   // mc = mm * 256 + c
    const int hg = g4 * kHeadsPerGroup + r;
    if (hg < G)
      lut[lay.off_exact + ((size_t)b * Hq + kv * G + hg) * ENTRIES + mc] =
          s_t[(r * M + mc / kCentroids) * ROW + (mc % kCentroids)];
  }
}

hipError_t launch_build_lut(const a2ats_dims& d, const void* q, int q_dtype, const float* cos_b,
                            const float* sin_b, const float* codebook, float* q_rot, int32_t* lut,
                            float* lut_scale, hipStream_t stream) {
  const int G = d.n_q_heads / d.n_kv_heads;
  const int NG = (G + kHeadsPerGroup - 1) / kHeadsPerGroup;
  const dim3 grid(d.batch * d.n_kv_heads * NG), block(kLutThreads);
  if (grid.x == 0) return hipSuccess;
  const size_t lds = (size_t)kHeadsPerGroup * d.n_sub * (kCentroids + 1) * sizeof(int32_t);
  static size_t s_slot[4][16];
  hipError_t err;
#define A2ATS_LAUNCH_LUT(DS, BF, SLOT)                                                              \
  do {                                                                                               \
    if ((err = allow_dynamic_lds(build_lut_kernel<DS, BF>, lds, s_slot[SLOT])) != hipSuccess) return err; \
    hipLaunchKernelGGL((build_lut_kernel<DS, BF>), grid, block, lds, stream, q, cos_b, sin_b, codebook, \
                       q_rot, lut, lut_scale, d.batch, d.n_q_heads, d.n_kv_heads, NG);               \
  } while (0)
  if (d.sub_dim == 8) {
    if (q_dtype == A2ATS_BF16) A2ATS_LAUNCH_LUT(8, true, 0); else A2ATS_LAUNCH_LUT(8, false, 1);
  } else {
    if (q_dtype == A2ATS_BF16) A2ATS_LAUNCH_LUT(4, true, 2); else A2ATS_LAUNCH_LUT(4, false, 3);
  }
#undef A2ATS_LAUNCH_LUT
  return hipGetLastError();
}

}  // namespace a2ats
