// The paper's own vector-quantisation geometry (section 5.1): ONE codebook of 4096 codewords per
// head over all D = 128 dimensions (M = 1), a 16-bit code per token.  The approximate score of a
// token is then a single table entry, u^_j = q~ . C[s_j] (section 2.2 eq. "attention weights
// approximation", section 4.2 last equation), so the code stream is 2 bytes per token and there
// are at most 4096 distinct scores per head: selection is dominated by exact ties.
//
//   build_lut_single_kernel    q~ = q R_b and the 4096 scores q~ . c per head, float64 inner
//                              products rounded once to float32 and stored as order-preserving
//                              32-bit keys (no fixed-point scale is needed: a score is one entry)
//   select_single_kernel       exact top-K per head: MSB-first radix select over the keys by
//                              re-streaming the codes, then one ordered pass that emits the winners
//                              in ascending position, equal scores going to the lower position
//   encode_single_*            query-aware assignment argmin_c (k - c) H (k - c)^T with the full
//                              D x D matrix H through its Cholesky factor (section 4.2)
#include "common.hpp"
#include "internal.hpp"

namespace a2ats {

constexpr int kCodewords = 4096;
constexpr int kSD = 128;   // head dimension = subspace dimension

// float32 score <-> signed 32-bit key with the same order (so that the integer selection
// machinery of the product-quantised path applies unchanged).
__device__ __forceinline__ int32_t float_to_key(float f) {
  const int32_t b = __float_as_int(f);
  return b ^ ((b >> 31) & 0x7fffffff);
}
__device__ __forceinline__ float key_to_float(int32_t k) {
  return __int_as_float(k ^ ((k >> 31) & 0x7fffffff));
}

// ------------------------------------------------------------------------------------------
// Tables
// ------------------------------------------------------------------------------------------
constexpr int kLutChunk = 256;   // codewords per workgroup

template <bool QBF16>
__global__ __launch_bounds__(kLutChunk) void build_lut_single_kernel(
    const void* __restrict__ q_in, const float* __restrict__ cos_b, const float* __restrict__ sin_b,
    const float* __restrict__ codebook, float* __restrict__ q_rot, int32_t* __restrict__ lut,
    float* __restrict__ lut_scale, int Hq, int Hkv) {
  constexpr int HALF = kSD / 2;
  __shared__ float s_q[8][kSD];   // q~ of the (up to) 8 query heads of this KV head
  const int chunk = blockIdx.x, bkv = blockIdx.y, b = bkv / Hkv, kv = bkv % Hkv;
  const int G = Hq / Hkv, tid = threadIdx.x;
  for (int i = tid; i < G * HALF; i += kLutChunk) {
    const int g = i / HALF, t = i % HALF;
    const size_t base = ((size_t)b * Hq + kv * G + g) * kSD;
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
    const float o1 = (float)(x1 * c - x2 * s), o2 = (float)(x2 * c + x1 * s);
    s_q[g][t] = o1;
    s_q[g][t + HALF] = o2;
    if (chunk == 0) {
      q_rot[base + t] = o1;
      q_rot[base + t + HALF] = o2;
      if (t == 0) lut_scale[(size_t)b * Hq + kv * G + g] = 1.f;
    }
  }
  __syncthreads();
  const int c = chunk * kLutChunk + tid;
  const float4* cw = (const float4*)(codebook + ((size_t)kv * kCodewords + c) * kSD);
  double acc[8];
#pragma unroll
  for (int g = 0; g < 8; ++g) acc[g] = 0.0;
#pragma unroll 4
  for (int t4 = 0; t4 < kSD / 4; ++t4) {
    const float4 f = cw[t4];
#pragma unroll
    for (int g = 0; g < 8; ++g) {
      if (g < G) {
        acc[g] += (double)s_q[g][4 * t4] * (double)f.x + (double)s_q[g][4 * t4 + 1] * (double)f.y +
                  (double)s_q[g][4 * t4 + 2] * (double)f.z + (double)s_q[g][4 * t4 + 3] * (double)f.w;
      }
    }
  }
#pragma unroll
  for (int g = 0; g < 8; ++g)
    if (g < G) lut[((size_t)b * Hq + kv * G + g) * kCodewords + c] = float_to_key((float)acc[g]);
}

hipError_t launch_build_lut_single(const a2ats_dims& d, const void* q, int q_dtype, const float* cos_b,
                                   const float* sin_b, const float* codebook, float* q_rot, int32_t* lut,
                                   float* lut_scale, hipStream_t stream) {
  const dim3 grid(kCodewords / kLutChunk, d.batch * d.n_kv_heads), block(kLutChunk);
  if (grid.y == 0) return hipSuccess;
  if (q_dtype == A2ATS_BF16)
    hipLaunchKernelGGL((build_lut_single_kernel<true>), grid, block, 0, stream, q, cos_b, sin_b, codebook,
                       q_rot, lut, lut_scale, d.n_q_heads, d.n_kv_heads);
  else
    hipLaunchKernelGGL((build_lut_single_kernel<false>), grid, block, 0, stream, q, cos_b, sin_b, codebook,
                       q_rot, lut, lut_scale, d.n_q_heads, d.n_kv_heads);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// Selection
// ------------------------------------------------------------------------------------------
constexpr int kSelThreads = 1024;
constexpr int kPerThread = 8;                       // consecutive tokens per thread and round
constexpr int kRound = kSelThreads * kPerThread;    // tokens per round

struct SelLds {
  int32_t table[kCodewords];
  uint32_t hist[kHistBins];
  uint32_t wave_a[kSelThreads / 64];
  uint32_t wave_b[kSelThreads / 64];
  uint32_t res[2];
  uint32_t kmin, kmax;
};

// The keys of tokens [j0, j0 + 8) of a sequence (positions at or past `hi` and before `lo` get
// `valid` false).  16-byte load when the row of codes allows it.
__device__ __forceinline__ void load_keys8(const uint16_t* __restrict__ seq_codes, bool aligned, int j0,
                                           int lo, int hi, const int32_t* table, uint32_t (&key)[kPerThread],
                                           bool (&valid)[kPerThread]) {
  uint16_t c[kPerThread];
  if (aligned && j0 >= 0 && j0 + kPerThread <= hi) {
    const uint4 v = *(const uint4*)(seq_codes + j0);
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < kPerThread; ++i) c[i] = (uint16_t)(w[i >> 1] >> (16 * (i & 1)));
  } else {
#pragma unroll
    for (int i = 0; i < kPerThread; ++i) {
      const int j = j0 + i;
      c[i] = (j >= 0 && j < hi) ? seq_codes[j] : (uint16_t)0;
    }
  }
#pragma unroll
  for (int i = 0; i < kPerThread; ++i) {
    const int j = j0 + i;
    valid[i] = j >= lo && j < hi;
    key[i] = score_key(table[c[i] & (kCodewords - 1)]);   // the mask keeps a bad code inside the table
  }
}

__global__ __launch_bounds__(kSelThreads) void select_single_kernel(
    const uint16_t* __restrict__ codes, const int32_t* __restrict__ lut, const int32_t* __restrict__ seq_lens,
    int32_t* __restrict__ topk_idx, int32_t* __restrict__ topk_count, float* __restrict__ topk_score,
    int Hq, int Hkv, int ctx_len, int64_t ctx_stride, int top_k, int window, int n_sink) {
  constexpr int NT = kSelThreads;
  __shared__ SelLds L;
  const int bh = blockIdx.x, b = bh / Hq, h = bh % Hq, G = Hq / Hkv, kv = h / G, tid = threadIdx.x;
  const SeqRange sr = seq_range(ctx_len, seq_lens, b, window, n_sink, top_k);
  int32_t* oi = topk_idx + (size_t)bh * top_k;
  float* os = topk_score ? topk_score + (size_t)bh * top_k : nullptr;
  if (tid == 0) topk_count[bh] = sr.kk;
  for (int t = sr.kk + tid; t < top_k; t += NT) {
    oi[t] = -1;
    if (os) os[t] = 0.f;
  }
  if (sr.kk == 0) return;

  const int32_t* head_table = lut + (size_t)bh * kCodewords;
  uint32_t kmin = 0xffffffffu, kmax = 0u;
  for (int e = tid; e < kCodewords; e += NT) {
    const int32_t v = head_table[e];
    L.table[e] = v;
    kmin = min(kmin, score_key(v));
    kmax = max(kmax, score_key(v));
  }
  if (tid == 0) {
    L.kmin = 0xffffffffu;
    L.kmax = 0u;
  }
  __syncthreads();
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    kmin = min(kmin, __shfl_xor(kmin, off));
    kmax = max(kmax, __shfl_xor(kmax, off));
  }
  if ((tid & 63) == 0) {
    atomicMin(&L.kmin, kmin);
    atomicMax(&L.kmax, kmax);
  }
  __syncthreads();
  const uint32_t k_lo = L.kmin;

  const uint16_t* seq_codes = codes + ((size_t)b * Hkv + kv) * ctx_stride;
  const bool aligned = (((uintptr_t)seq_codes) & 15u) == 0;
  const int lo = sr.sink_end, hi = sr.win_start;
  const int first = lo & ~(kPerThread - 1);   // rounds start on a multiple of 8 tokens

  uint32_t kth = 0, k_rem = (uint32_t)sr.kk;
  if (sr.kk < sr.ncand) {
    // Radix digits are taken from key - smallest key of the table, MSB first.
    int remaining = 32 - __clz(L.kmax - k_lo);
    uint32_t prefix = 0, mask = 0;
#pragma unroll 1
    while (remaining > 0) {
      const int bits = remaining < 11 ? remaining : 11;
      const int shift = remaining - bits;
      const uint32_t dmask = (1u << bits) - 1u;
      for (int i = tid; i < kHistBins; i += NT) L.hist[i] = 0;
      __syncthreads();
      for (int base = first; base < hi; base += kRound) {
        uint32_t key[kPerThread];
        bool valid[kPerThread];
        load_keys8(seq_codes, aligned, base + tid * kPerThread, lo, hi, L.table, key, valid);
#pragma unroll
        for (int i = 0; i < kPerThread; ++i) {
          const uint32_t rel = key[i] - k_lo;
          if (valid[i] && (rel & mask) == prefix) atomicAdd(&L.hist[(rel >> shift) & dmask], 1u);
        }
      }
      __syncthreads();
      block_find_rank_desc<NT, kHistBins>([&](int i) { return L.hist[i]; }, k_rem, L.wave_a, L.res);
      const uint32_t bin = L.res[0], above = L.res[1];
      k_rem -= above;
      prefix |= bin << shift;
      mask |= dmask << shift;
      remaining = shift;
      __syncthreads();
    }
    kth = prefix + k_lo;
  }

  // Ordered emission: keys above the K-th, plus the first k_rem positions that equal it.  A thread
  // owns 8 consecutive positions, so one scan of packed (above, equal) counts per round places
  // every winner.
  const bool take_all = sr.kk >= sr.ncand;
  uint32_t out_n = 0, eq_seen = 0;
#pragma unroll 1
  for (int base = first; base < hi; base += kRound) {
    uint32_t key[kPerThread];
    bool valid[kPerThread];
    const int j0 = base + tid * kPerThread;
    load_keys8(seq_codes, aligned, j0, lo, hi, L.table, key, valid);
    uint32_t loc = 0;
#pragma unroll
    for (int i = 0; i < kPerThread; ++i) {
      const bool gt = valid[i] && (take_all || key[i] > kth);
      const bool eq = valid[i] && !take_all && key[i] == kth;
      loc += (gt ? 1u : 0u) + (eq ? 0x10000u : 0u);
    }
    uint32_t tot;
    uint32_t pre = block_exclusive_scan<NT>(loc, (base / kRound) & 1 ? L.wave_b : L.wave_a, tot);
    uint32_t gt_before = pre & 0xffffu, eq_before = eq_seen + (pre >> 16);
#pragma unroll
    for (int i = 0; i < kPerThread; ++i) {
      const bool gt = valid[i] && (take_all || key[i] > kth);
      const bool eq = valid[i] && !take_all && key[i] == kth;
      if (gt || (eq && eq_before < k_rem)) {
        const uint32_t slot = out_n + gt_before + min(eq_before, k_rem);
        oi[slot] = j0 + i;
        if (os) os[slot] = key_to_float(key_score(key[i]));
      }
      gt_before += gt ? 1u : 0u;
      eq_before += eq ? 1u : 0u;
    }
    out_n += tot & 0xffffu;
    eq_seen += tot >> 16;
    if (out_n + min(eq_seen, k_rem) >= (uint32_t)sr.kk) break;   // uniform: tot is the block total
  }
}

// Debug / parity: every token's score as float.
__global__ __launch_bounds__(256) void score_dense_single_kernel(
    const uint16_t* __restrict__ codes, const int32_t* __restrict__ lut, const int32_t* __restrict__ seq_lens,
    float* __restrict__ scores_out, int Hq, int Hkv, int ctx_len, int64_t ctx_stride) {
  const int bh = blockIdx.y, b = bh / Hq, h = bh % Hq, G = Hq / Hkv, kv = h / G;
  int n = seq_lens ? seq_lens[b] : ctx_len;
  n = n < 0 ? 0 : (n > ctx_len ? ctx_len : n);
  const uint16_t* seq_codes = codes + ((size_t)b * Hkv + kv) * ctx_stride;
  const int32_t* table = lut + (size_t)bh * kCodewords;
  for (int j = blockIdx.x * 256 + threadIdx.x; j < n; j += gridDim.x * 256)
    scores_out[(size_t)bh * ctx_stride + j] = key_to_float(table[seq_codes[j] & (kCodewords - 1)]);
}

hipError_t launch_score_topk_single(const a2ats_dims& d, const void* codes, const int32_t* lut, int top_k,
                                    int window, int n_sink, const int32_t* seq_lens, int32_t* topk_idx,
                                    int32_t* topk_count, float* topk_score, float* scores_out,
                                    hipStream_t stream) {
  const int heads = d.batch * d.n_q_heads;
  if (heads == 0) return hipSuccess;
  if (scores_out) {
    int gx = (d.ctx_len + 256 * 8 - 1) / (256 * 8);
    if (gx < 1) gx = 1;
    hipLaunchKernelGGL(score_dense_single_kernel, dim3(gx, heads), dim3(256), 0, stream,
                       (const uint16_t*)codes, lut, seq_lens, scores_out, d.n_q_heads, d.n_kv_heads,
                       d.ctx_len, d.ctx_stride);
    const hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
  }
  hipLaunchKernelGGL(select_single_kernel, dim3(heads), dim3(kSelThreads), 0, stream, (const uint16_t*)codes,
                     lut, seq_lens, topk_idx, topk_count, topk_score, d.n_q_heads, d.n_kv_heads, d.ctx_len,
                     d.ctx_stride, top_k, window, n_sink);
  return hipGetLastError();
}

}  // namespace a2ats
