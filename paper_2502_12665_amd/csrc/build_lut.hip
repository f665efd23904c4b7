// Steps 1-2 of a decode step: WRoPE query rotation (section 4.1: q~ = q R_b) and the
// per-subspace query x centroid tables (section 4.2 last equation, tabulated per subspace).
//
// One workgroup per (sequence, KV head, group of 4 query heads).  The contraction is
// 2*B*Hq*256*D flop in total (8.4 Mflop at the 131072-token configuration), far below
// anything a matrix core would help with, so it runs on the vector ALU in float64: products
// of two float32 values are exact in float64, which makes every table entry the correctly
// rounded inner product.  Three things are written per head (see "Lookup-table format" in
// a2ats.h): the exact 32-bit fixed-point table [c][m], a 16-bit coarse copy of it interleaved
// over the four heads of the group [c][m][4] for the streaming kernel, and the numbers that
// relate them (sum of the per-subspace minima, shift, sum of the per-subspace maxima).
#include "common.hpp"
#include "internal.hpp"
#include "encode_few.hpp"
#include "coarse_score.hpp"

namespace a2ats {

constexpr int kLutThreads = 1024;

// SHARED: one table per KV head, built from the sum of the rotated queries of its G heads (the
// group's summed score sum_g q~_g . c equals (sum_g q~_g) . c); the rotated queries themselves
// are still written per head.  The table array is then laid out as for n_q_heads == n_kv_heads.
template <int DS, bool QBF16, bool SHARED = false>
__device__ __forceinline__ void build_lut_body(
    int prob, const void* __restrict__ q_in, const float* __restrict__ cos_b,
    const float* __restrict__ sin_b, const float* __restrict__ codebook, float* __restrict__ q_rot,
    int32_t* __restrict__ lut, float* __restrict__ lut_scale, int B, int Hq, int Hkv, int NG,
    bool write_out = true, unsigned char* coarse_lds = nullptr) {
  // write_out false: the tables are computed but nothing is written to global memory (another
  // workgroup does that); coarse_lds: the group's coarse table is also put there, in the layout the
  // scoring kernels read (one 256-byte row per centroid id).
  constexpr int D = 128, HALF = 64, M = D / DS;
  constexpr int ENTRIES = kCentroids * M;
  constexpr int EPT = ENTRIES / kLutThreads;
  constexpr int MAXQ = 65535 / M;       // a sum of M coarse entries fits 16 bits
  constexpr int LOG2M = M == 16 ? 4 : 5;
  static_assert(M == 16 || M == 32, "M is 16 or 32");
  __shared__ float s_q[kHeadsPerGroup][D];
  __shared__ uint32_t s_maxbits[kHeadsPerGroup];   // largest |entry| per head, as float bits
  __shared__ int32_t s_min[M][kHeadsPerGroup], s_max[M][kHeadsPerGroup];
  __shared__ int32_t s_shift[kHeadsPerGroup];

  const int Gq = Hq / Hkv;                 // query heads per KV head
  const int G = SHARED ? 1 : Gq;           // table heads per KV head
  const int Hq_q = Hq;
  if (SHARED) Hq = Hkv;                    // table indexing below is per table head
  const int g4 = prob % NG, kv = (prob / NG) % Hkv, b = prob / (NG * Hkv);
  const int tid = threadIdx.x;
  const LutLayout lay = lut_layout(B, Hq, Hkv, M);

  // The codebook rows of this thread's entries (e = c * M + m, so its entries share m = tid % M)
  // are requested first: their latency overlaps the query rotation.
  const int m = tid % M;
  float cv[EPT][DS];
#pragma unroll
  for (int k = 0; k < EPT; ++k) {
    const int c = (tid + k * kLutThreads) / M;
    const float* cw = codebook + (((size_t)kv * M + m) * kCentroids + c) * DS;
#pragma unroll
    for (int t = 0; t < DS; t += 4) {
      const float4 f = *(const float4*)(cw + t);
      cv[k][t] = f.x; cv[k][t + 1] = f.y; cv[k][t + 2] = f.z; cv[k][t + 3] = f.w;
    }
  }

  // --- q~ = q R_b for the (up to) four heads of this group (SHARED: all G <= 8 heads of the KV head)
  __shared__ float s_qall[SHARED ? 8 : 1][SHARED ? D : 1];
  if (tid < (SHARED ? 8 : kHeadsPerGroup) * HALF) {
    const int r = tid / HALF, t = tid % HALF;
    const int hg = SHARED ? r : g4 * kHeadsPerGroup + r;
    float o1 = 0.f, o2 = 0.f;
    if (hg < Gq) {
      const int h = kv * Gq + hg;
      const size_t base = ((size_t)b * Hq_q + h) * D;
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
      if (write_out) {
        q_rot[base + t] = o1;
        q_rot[base + t + HALF] = o2;
      }
    }
    if (SHARED) {
      s_qall[r][t] = o1;
      s_qall[r][t + HALF] = o2;
    } else {
      s_q[r][t] = o1;
      s_q[r][t + HALF] = o2;
    }
  }
  if (SHARED) {
    __syncthreads();
    if (tid < kHeadsPerGroup * D) {
      const int r = tid / D, t = tid % D;
      double sum = 0.0;
      if (r == 0)
        for (int g = 0; g < 8; ++g) sum += (double)s_qall[g][t];   // heads past G hold zeros
      s_q[r][t] = (float)sum;
    }
  }
  if (tid < kHeadsPerGroup) s_maxbits[tid] = 0u;
  if (tid < M * kHeadsPerGroup) {
    s_min[tid / kHeadsPerGroup][tid % kHeadsPerGroup] = INT32_MAX;
    s_max[tid / kHeadsPerGroup][tid % kHeadsPerGroup] = INT32_MIN;
  }
  __syncthreads();

  // --- table entries in float64
  double val[EPT][kHeadsPerGroup];
  double mxd[kHeadsPerGroup] = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
  for (int k = 0; k < EPT; ++k) {
#pragma unroll
    for (int r = 0; r < kHeadsPerGroup; ++r) {
      double acc = 0.0;
#pragma unroll
      for (int t = 0; t < DS; ++t) acc += (double)s_q[r][m * DS + t] * (double)cv[k][t];
      val[k][r] = acc;
      mxd[r] = fmax(mxd[r], fabs(acc));
    }
  }
  // The thread's maximum as a float rounded up, so that it is never below the true one (rounding is
  // monotone: the same number as the maximum of the rounded entries, with one change of the rounding
  // mode per head instead of one per entry).
  float mx[kHeadsPerGroup];
#pragma unroll
  for (int r = 0; r < kHeadsPerGroup; ++r) mx[r] = __double2float_ru(mxd[r]);

  // --- per-head power-of-two scale: M * max|entry| * 2^e < 2^30.  Non-negative floats order like
  // their bit patterns, so the block maximum is an integer atomic max in LDS (one per wave and head
  // after a reduction over the wave).
#pragma unroll
  for (int r = 0; r < kHeadsPerGroup; ++r) {
    const uint32_t v = wave_max_to_last_lane(__float_as_uint(mx[r]));
    if ((tid & 63) == 63) atomicMax(&s_maxbits[r], v);
  }
  __syncthreads();
  // Every thread derives the four exponents itself (M is a power of two and v a float, so the
  // exponent of v * M is the float's exponent field plus a constant; a subnormal maximum takes the
  // general route): no second barrier, no double-precision library call on the critical path.
  int s_exp[kHeadsPerGroup];
#pragma unroll
  for (int r = 0; r < kHeadsPerGroup; ++r) {
    const uint32_t bits = s_maxbits[r];
    int e = 0;
    if (bits != 0u) {
      int x;   // v * M < 2^x
      if ((bits >> 23) != 0u) {
        x = (int)(bits >> 23) - 126 + LOG2M;
      } else {
        frexp((double)__uint_as_float(bits) * (double)M, &x);
      }
      e = 30 - x;
      e = e > 100 ? 100 : (e < -100 ? -100 : e);
    }
    s_exp[r] = e;
  }
  if (tid < kHeadsPerGroup) {
    const int hg = g4 * kHeadsPerGroup + tid;
    if (hg < G && write_out) lut_scale[(size_t)b * Hq + kv * G + hg] = (float)ldexp(1.0, -s_exp[tid]);
  }

  // --- exact fixed-point entries; per-(subspace, head) minimum and maximum over the centroids
  // (LDS atomics: the four lanes of a wave that share a subspace collide, nothing else does)
  int32_t iv[EPT][kHeadsPerGroup];
  {
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
    for (int r = 0; r < kHeadsPerGroup; ++r) {
      atomicMin(&s_min[m][r], mn[r]);
      atomicMax(&s_max[m][r], mxv[r]);
    }
  }
  __syncthreads();
  if (tid < kHeadsPerGroup) {
    const int r = tid;
    uint32_t range = 0;
    int32_t base = 0, top = 0;
    for (int mm = 0; mm < M; ++mm) {
      range = max(range, (uint32_t)(s_max[mm][r] - s_min[mm][r]));
      base += s_min[mm][r];
      top += s_max[mm][r];
    }
    int sh = 0;
    while ((range >> sh) > (uint32_t)MAXQ) ++sh;
    s_shift[r] = sh;
    const int hg = g4 * kHeadsPerGroup + r;
    if (hg < G && write_out) {
      int32_t* meta = lut + lay.off_meta + ((size_t)b * Hq + kv * G + hg) * 4;
      meta[0] = base;   // sum over subspaces of the smallest entry
      meta[1] = sh;     // coarse entry = (exact entry - subspace minimum) >> sh
      meta[2] = top;    // sum over subspaces of the largest entry: no score exceeds it
      meta[3] = 0;
    }
  }
  // --- exact tables, one per head as [c][m]: entry e of a thread is word e of the head's table
#pragma unroll
  for (int r = 0; r < kHeadsPerGroup; ++r) {
    const int hg = g4 * kHeadsPerGroup + r;
    if (hg < G && write_out) {
      int32_t* ex = lut + lay.off_exact + ((size_t)b * Hq + kv * G + hg) * ENTRIES;
#pragma unroll
      for (int k = 0; k < EPT; ++k) ex[tid + k * kLutThreads] = iv[k][r];
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
      const uint2 entry = make_uint2(q0 | (q1 << 16), q2 | (q3 << 16));
      if (write_out) coarse[(m >> 4) * (kCentroids * 16) + c * 16 + (m & 15)] = entry;
      if (coarse_lds) store_coarse_lds<M>(coarse_lds, c, m, entry);
    }
  }
}

template <int DS, bool QBF16>
__global__ __launch_bounds__(kLutThreads) void build_lut_kernel(
    const void* __restrict__ q_in, const float* __restrict__ cos_b, const float* __restrict__ sin_b,
    const float* __restrict__ codebook, float* __restrict__ q_rot, int32_t* __restrict__ lut,
    float* __restrict__ lut_scale, int B, int Hq, int Hkv, int NG) {
  build_lut_body<DS, QBF16>(blockIdx.x, q_in, cos_b, sin_b, codebook, q_rot, lut, lut_scale, B, Hq, Hkv, NG);
}

template <int DS, bool QBF16>
__global__ __launch_bounds__(kLutThreads) void build_lut_shared_kernel(
    const void* __restrict__ q_in, const float* __restrict__ cos_b, const float* __restrict__ sin_b,
    const float* __restrict__ codebook, float* __restrict__ q_rot, int32_t* __restrict__ lut,
    float* __restrict__ lut_scale, int B, int Hq, int Hkv) {
  build_lut_body<DS, QBF16, true>(blockIdx.x, q_in, cos_b, sin_b, codebook, q_rot, lut, lut_scale, B, Hq, Hkv, 1);
}

// An encoding workgroup of the prologues below: wave w takes the pairs (block * sweeps + s) * 16 + w.
template <int DS>
__device__ __forceinline__ void encode_few_block(int block, int sweeps, const float* __restrict__ keys,
                                                 const float* __restrict__ codebook,
                                                 const float* __restrict__ weights, int mode,
                                                 uint8_t* __restrict__ codes, int B, int Hkv, int n_new, int pos0,
                                                 int64_t ctx_stride) {
  constexpr int M = 128 / DS;
  static_assert(kLutThreads / 64 == kFewPairsPerSweep, "one pair per wave and sweep");
  const long n_pairs = (long)B * Hkv * n_new * M;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  for (int s = 0; s < sweeps; ++s) {
    const long pair = ((long)block * sweeps + s) * kFewPairsPerSweep + wave;
    if (pair < n_pairs)   // (uniform over the wave)
      encode_few_wave<DS>(keys, codebook, weights, mode, codes, Hkv, M, n_new, pos0, ctx_stride, pair, lane);
  }
}

// Decode prologue in one launch: the first n_lut workgroups build the tables of the current query,
// the others encode the few keys appended this step, one (key, subspace) pair per wave and sweep.
// The two halves touch disjoint data.  The kernel holds one workgroup per CU, so when the two kinds
// together would not fit one round of the CUs the launch is "folded": no encoding workgroups, the
// table workgroups share the pairs out among themselves.
template <int DS, bool QBF16>
__global__ __launch_bounds__(kLutThreads) void decode_prologue_kernel(
    const void* __restrict__ q_in, const float* __restrict__ cos_b, const float* __restrict__ sin_b,
    const float* __restrict__ codebook, float* __restrict__ q_rot, int32_t* __restrict__ lut,
    float* __restrict__ lut_scale, int B, int Hq, int Hkv, int NG, int n_lut,
    const float* __restrict__ keys, const float* __restrict__ weights, int mode,
    uint8_t* __restrict__ codes, int n_new, int pos0, int64_t ctx_stride, int sweeps, int folded) {
  if ((int)blockIdx.x < n_lut) {
    build_lut_body<DS, QBF16>(blockIdx.x, q_in, cos_b, sin_b, codebook, q_rot, lut, lut_scale, B, Hq, Hkv, NG);
    // folded: the table workgroups encode as well, after their stores have been issued (their tail
    // waits for those to drain anyway)
    if (folded)
      encode_few_block<DS>((int)blockIdx.x, sweeps, keys, codebook, weights, mode, codes, B, Hkv, n_new, pos0,
                           ctx_stride);
    return;
  }
  encode_few_block<DS>((int)blockIdx.x - n_lut, sweeps, keys, codebook, weights, mode, codes, B, Hkv, n_new, pos0,
                       ctx_stride);
}

// The decode prologue and the first launch of a2ats_score_topk's streaming route in one: every
// sampling workgroup (P0 per problem) builds its problem's tables itself -- the arithmetic is a few
// microseconds and identical in all of them -- keeps the coarse table in LDS and scores its share of
// the sample against it; part 0 of a problem also writes the tables out for the launches that
// follow.  The remaining workgroups encode the appended keys.  Saves one launch and the copy of the
// table from global memory per step; every result is bit for bit that of the separate calls.
// SHARED: one table per KV head from the summed rotated queries of its heads (build_lut_body<.., true>);
// the thresholds are then per KV head (NG is 1 and the sampling sees Hkv table heads).
template <int DS, bool QBF16, bool SHARED>
__global__ __launch_bounds__(kLutThreads) void decode_select_prologue_kernel(
    const void* __restrict__ q_in, const float* __restrict__ cos_b, const float* __restrict__ sin_b,
    const float* __restrict__ codebook, float* __restrict__ q_rot, int32_t* __restrict__ lut,
    float* __restrict__ lut_scale, int B, int Hq, int Hkv, int NG, int n_sample,
    const float* __restrict__ keys, const float* __restrict__ weights, int mode,
    uint8_t* __restrict__ codes, int n_new, int pos0, int64_t ctx_stride,
    const int32_t* __restrict__ seq_lens, int32_t* __restrict__ thr, int P0, int sample_rows, int ctx_len,
    int top_k, int window, int n_sink, int sweeps) {
  constexpr int M = 128 / DS;
  extern __shared__ __align__(16) unsigned char dyn_lds[];
  if ((int)blockIdx.x < n_sample) {
    int prob, p;
    xcd_map_sets(blockIdx.x, P0, n_sample / P0, NG, prob, p);
    build_lut_body<DS, QBF16, SHARED>(prob, q_in, cos_b, sin_b, codebook, q_rot, lut, lut_scale, B, Hq, Hkv, NG,
                                      p == 0, dyn_lds);
    __syncthreads();
    sample_threshold_body<M, kLutThreads, true>(prob, p, codes, CodePages{nullptr, 0, 0}, lut, seq_lens, thr, B,
                                                SHARED ? Hkv : Hq, Hkv, NG, P0, sample_rows, ctx_len, ctx_stride,
                                                top_k, window, n_sink, dyn_lds);
    return;
  }
  encode_few_block<DS>((int)blockIdx.x - n_sample, sweeps, keys, codebook, weights, mode, codes, B, Hkv, n_new, pos0,
                       ctx_stride);
}

hipError_t launch_decode_select_prologue(const a2ats_dims& d, const float* keys, int n_new, int pos0,
                                         const float* codebook, const float* weights, int mode, uint8_t* codes,
                                         const void* q, int q_dtype, const float* cos_b, const float* sin_b,
                                         float* q_rot, int32_t* lut, float* lut_scale, const int32_t* seq_lens,
                                         int32_t* thr, int P0, int sample_rows, int top_k, int window, int n_sink,
                                         bool shared, hipStream_t stream) {
  const int G = d.n_q_heads / d.n_kv_heads;
  const int NG = shared ? 1 : (G + kHeadsPerGroup - 1) / kHeadsPerGroup;
  const int n_sample = d.batch * d.n_kv_heads * NG * P0;
  const long n_pairs = (long)d.batch * d.n_kv_heads * n_new * d.n_sub;
  const int sweeps = encode_few_sweeps(n_pairs);
  const long per_wg = (long)kFewPairsPerSweep * sweeps;
  const dim3 grid(n_sample + (unsigned)((n_pairs + per_wg - 1) / per_wg)), block(kLutThreads);
  if (grid.x == 0) return hipSuccess;
  static LdsSlot s_lds[8][16];
  hipError_t err;
#define A2ATS_LAUNCH_SEL(DS, BF, SH, SLOT)                                                                   \
  do {                                                                                                       \
    if ((err = allow_dynamic_lds(decode_select_prologue_kernel<DS, BF, SH>, (size_t)kCoarseLdsBytes,         \
                                 s_lds[SLOT])) != hipSuccess)                                                \
      return err;                                                                                            \
    hipLaunchKernelGGL((decode_select_prologue_kernel<DS, BF, SH>), grid, block, kCoarseLdsBytes, stream, q, \
                       cos_b, sin_b, codebook, q_rot, lut, lut_scale, d.batch, d.n_q_heads, d.n_kv_heads, NG, \
                       n_sample, keys, weights, mode, codes, n_new, pos0, d.ctx_stride, seq_lens, thr, P0,   \
                       sample_rows, d.ctx_len, top_k, window, n_sink, sweeps);                               \
  } while (0)
#define A2ATS_LAUNCH_SEL2(DS, BF, SLOT)                                    \
  do {                                                                     \
    if (shared) A2ATS_LAUNCH_SEL(DS, BF, true, SLOT + 4);                  \
    else A2ATS_LAUNCH_SEL(DS, BF, false, SLOT);                            \
  } while (0)
  if (d.sub_dim == 8) {
    if (q_dtype == A2ATS_BF16) A2ATS_LAUNCH_SEL2(8, true, 0); else A2ATS_LAUNCH_SEL2(8, false, 1);
  } else {
    if (q_dtype == A2ATS_BF16) A2ATS_LAUNCH_SEL2(4, true, 2); else A2ATS_LAUNCH_SEL2(4, false, 3);
  }
#undef A2ATS_LAUNCH_SEL2
#undef A2ATS_LAUNCH_SEL
  return hipGetLastError();
}

hipError_t launch_build_lut(const a2ats_dims& d, const void* q, int q_dtype, const float* cos_b,
                            const float* sin_b, const float* codebook, float* q_rot, int32_t* lut,
                            float* lut_scale, hipStream_t stream) {
  const int G = d.n_q_heads / d.n_kv_heads;
  const int NG = (G + kHeadsPerGroup - 1) / kHeadsPerGroup;
  const dim3 grid(d.batch * d.n_kv_heads * NG), block(kLutThreads);
  if (grid.x == 0) return hipSuccess;
#define A2ATS_LAUNCH_LUT(DS, BF)                                                                    \
  hipLaunchKernelGGL((build_lut_kernel<DS, BF>), grid, block, 0, stream, q, cos_b, sin_b, codebook, \
                     q_rot, lut, lut_scale, d.batch, d.n_q_heads, d.n_kv_heads, NG)
  if (d.sub_dim == 8) {
    if (q_dtype == A2ATS_BF16) A2ATS_LAUNCH_LUT(8, true); else A2ATS_LAUNCH_LUT(8, false);
  } else {
    if (q_dtype == A2ATS_BF16) A2ATS_LAUNCH_LUT(4, true); else A2ATS_LAUNCH_LUT(4, false);
  }
#undef A2ATS_LAUNCH_LUT
  return hipGetLastError();
}

hipError_t launch_build_lut_shared(const a2ats_dims& d, const void* q, int q_dtype, const float* cos_b,
                                   const float* sin_b, const float* codebook, float* q_rot, int32_t* lut,
                                   float* lut_scale, hipStream_t stream) {
  const dim3 grid(d.batch * d.n_kv_heads), block(kLutThreads);
  if (grid.x == 0) return hipSuccess;
#define A2ATS_LAUNCH_LUTS(DS, BF)                                                                          \
  hipLaunchKernelGGL((build_lut_shared_kernel<DS, BF>), grid, block, 0, stream, q, cos_b, sin_b, codebook, \
                     q_rot, lut, lut_scale, d.batch, d.n_q_heads, d.n_kv_heads)
  if (d.sub_dim == 8) {
    if (q_dtype == A2ATS_BF16) A2ATS_LAUNCH_LUTS(8, true); else A2ATS_LAUNCH_LUTS(8, false);
  } else {
    if (q_dtype == A2ATS_BF16) A2ATS_LAUNCH_LUTS(4, true); else A2ATS_LAUNCH_LUTS(4, false);
  }
#undef A2ATS_LAUNCH_LUTS
  return hipGetLastError();
}

hipError_t launch_decode_prologue(const a2ats_dims& d, const float* keys, int n_new, int pos0,
                                  const float* codebook, const float* weights, int mode, uint8_t* codes,
                                  const void* q, int q_dtype, const float* cos_b, const float* sin_b,
                                  float* q_rot, int32_t* lut, float* lut_scale, hipStream_t stream) {
  const int G = d.n_q_heads / d.n_kv_heads;
  const int NG = (G + kHeadsPerGroup - 1) / kHeadsPerGroup;
  const int n_lut = d.batch * d.n_kv_heads * NG;
  const long n_pairs = (long)d.batch * d.n_kv_heads * n_new * d.n_sub;
  int sweeps = encode_few_sweeps(n_pairs);
  long n_enc = (n_pairs + (long)kFewPairsPerSweep * sweeps - 1) / ((long)kFewPairsPerSweep * sweeps);
  const int folded = n_lut > 0 && n_lut + n_enc > 256;
  if (folded) {
    sweeps = (int)((n_pairs + (long)kFewPairsPerSweep * n_lut - 1) / ((long)kFewPairsPerSweep * n_lut));
    n_enc = 0;
  }
  const dim3 grid(n_lut + (unsigned)n_enc), block(kLutThreads);
  if (grid.x == 0) return hipSuccess;
#define A2ATS_LAUNCH_PRO(DS, BF)                                                                       \
  hipLaunchKernelGGL((decode_prologue_kernel<DS, BF>), grid, block, 0, stream, q, cos_b, sin_b, codebook, \
                     q_rot, lut, lut_scale, d.batch, d.n_q_heads, d.n_kv_heads, NG, n_lut, keys, weights, \
                     mode, codes, n_new, pos0, d.ctx_stride, sweeps, folded)
  if (d.sub_dim == 8) {
    if (q_dtype == A2ATS_BF16) A2ATS_LAUNCH_PRO(8, true); else A2ATS_LAUNCH_PRO(8, false);
  } else {
    if (q_dtype == A2ATS_BF16) A2ATS_LAUNCH_PRO(4, true); else A2ATS_LAUNCH_PRO(4, false);
  }
#undef A2ATS_LAUNCH_PRO
  return hipGetLastError();
}

}  // namespace a2ats
