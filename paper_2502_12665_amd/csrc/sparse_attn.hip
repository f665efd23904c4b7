// Step 4 of a decode step: exact attention over sinks U top-K U window under WRoPE
// (section 2.1 eq. "output state" restricted to the attended set; section 4.1 eq. "WRoPE").
//
// The phase is a random-row gather from HBM: per query head about K + w key rows and as many
// value rows of 256 B (bf16) or 512 B (float32) each, 2 flop per byte fetched.  Every query
// head has its own retrieved set, so the "matrix" on the query side has one row; the
// products are therefore done on the vector ALU and all effort goes into keeping many row
// loads in flight: a row is read by 16 (bf16) or 32 (float32) lanes with one 16-byte load
// each, a wave works on 4 (2) rows at a time, and the rows of one head are split over
// several workgroups whose partial (max, sum, accumulator) triples a second small kernel
// merges.
#include "common.hpp"
#include "internal.hpp"

namespace a2ats {

constexpr int kAttnThreads = 256;
constexpr int kAttnTile = 512;   // positions staged in LDS at a time
constexpr int kD = 128;

AttnPlan make_attn_plan(const a2ats_dims& d, int top_k, int window, int n_sink) {
  AttnPlan p;
  const long heads = (long)d.batch * d.n_q_heads;
  long rows = (long)n_sink + top_k + window;
  if (rows > d.ctx_len) rows = d.ctx_len;
  long ns = heads > 0 ? (1024 + heads - 1) / heads : 1;
  const long by_rows = rows / 64 > 1 ? rows / 64 : 1;
  if (ns > by_rows) ns = by_rows;
  if (ns > 32) ns = 32;
  if (ns < 1) ns = 1;
  p.n_split = (int)ns;
  p.bytes = ns > 1 ? (size_t)heads * ns * (kD + 2) * sizeof(float) : 0;
  return p;
}

template <typename T> struct RowVec;
template <> struct RowVec<float> {
  static constexpr int LPR = 32, VEC = 4;
  static __device__ __forceinline__ void load(const float* p, float (&o)[4]) {
    const float4 v = *(const float4*)p;
    o[0] = v.x; o[1] = v.y; o[2] = v.z; o[3] = v.w;
  }
};
template <> struct RowVec<uint16_t> {
  static constexpr int LPR = 16, VEC = 8;
  static __device__ __forceinline__ void load(const uint16_t* p, float (&o)[8]) {
    const uint4 v = *(const uint4*)p;
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      o[2 * i] = __uint_as_float(w[i] << 16);
      o[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
  }
};

__device__ __forceinline__ float load_elem(const float* p) { return *p; }
__device__ __forceinline__ float load_elem(const uint16_t* p) { return bf16_to_f32(*p); }
__device__ __forceinline__ void store_elem(float* p, float v) { *p = v; }
__device__ __forceinline__ void store_elem(uint16_t* p, float v) { *p = f32_to_bf16(v); }

// Merge two online-softmax states.
template <int VEC>
__device__ __forceinline__ void merge_state(float& m, float& l, float (&acc)[VEC], float m2, float l2,
                                            const float (&acc2)[VEC]) {
  const float mm = fmaxf(m, m2);
  if (mm == -INFINITY) return;
  const float s1 = __expf(m - mm), s2 = __expf(m2 - mm);
  l = l * s1 + l2 * s2;
#pragma unroll
  for (int v = 0; v < VEC; ++v) acc[v] = acc[v] * s1 + acc2[v] * s2;
  m = mm;
}

template <typename T>
__global__ __launch_bounds__(kAttnThreads) void attn_partial_kernel(
    const T* __restrict__ q, const float* __restrict__ q_rot, const T* __restrict__ k_cache,
    const T* __restrict__ v_cache, const int32_t* __restrict__ topk_idx,
    const int32_t* __restrict__ topk_count, const float* __restrict__ cos_win,
    const float* __restrict__ sin_win, const int32_t* __restrict__ seq_lens, T* __restrict__ out,
    float* __restrict__ partial, int Hq, int Hkv, int ctx_len, int64_t ctx_stride, int top_k,
    int window, int n_sink, int n_split) {
  constexpr int LPR = RowVec<T>::LPR, VEC = RowVec<T>::VEC;
  constexpr int SLOTS = 64 / LPR;            // rows a wave reads at once
  constexpr int NWV = kAttnThreads / 64;
  constexpr int RB = NWV * SLOTS;            // rows per block step
  constexpr int HALF = kD / 2;
  __shared__ int32_t s_pos[kAttnTile];
  __shared__ float s_m[NWV], s_l[NWV], s_acc[NWV][kD];

  const int split = blockIdx.x, bh = blockIdx.y, b = bh / Hq, h = bh % Hq;
  const int G = Hq / Hkv, kv = h / G;
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, slot = lane / LPR, sub = lane % LPR;
  const SeqRange sr = seq_range(ctx_len, seq_lens, b, window, n_sink, top_k);
  const int cnt = max(0, min(min(topk_count[bh], top_k), sr.ncand));
  const int n_att = sr.sink_end + cnt + (sr.n - sr.win_start);
  const int per = (n_att + n_split - 1) / n_split;
  const int t0 = split * per, t1 = min(n_att, t0 + per);

  // this lane's slice of the query: own dims d0..d0+VEC-1 and the dims paired with them
  const int d0 = sub * VEC;
  const bool low_half = d0 < HALF;
  const int dp = low_half ? d0 + HALF : d0 - HALF;
  const float sgn = low_half ? -1.f : 1.f;
  float q_own[VEC], q_par[VEC], q_far[VEC];
  {
    const size_t qb = (size_t)bh * kD;
#pragma unroll
    for (int v = 0; v < VEC; ++v) {
      q_own[v] = load_elem(q + qb + d0 + v);
      q_par[v] = load_elem(q + qb + dp + v) * sgn;
      q_far[v] = q_rot[qb + d0 + v];
    }
  }
  const float scale = 0.08838834764831845f;   // 1/sqrt(128)
  const T* kb = k_cache + ((size_t)b * Hkv + kv) * ctx_stride * kD + d0;
  const T* vb = v_cache + ((size_t)b * Hkv + kv) * ctx_stride * kD + d0;
  const int32_t* idx = topk_idx + (size_t)bh * top_k;

  float m_run = -INFINITY, l_run = 0.f, acc[VEC];
#pragma unroll
  for (int v = 0; v < VEC; ++v) acc[v] = 0.f;

  for (int tb = t0; tb < t1; tb += kAttnTile) {
    const int tn = min(kAttnTile, t1 - tb);
    __syncthreads();
    for (int i = tid; i < tn; i += kAttnThreads) {
      const int t = tb + i;
      int j;
      if (t < sr.sink_end) j = t;
      else if (t < sr.sink_end + cnt) j = idx[t - sr.sink_end];
      else j = sr.win_start + (t - sr.sink_end - cnt);
      s_pos[i] = min(max(j, 0), sr.n - 1);   // a bad caller index must not leave the cache
    }
    __syncthreads();
    constexpr int U = 2;
    for (int i0 = wv * SLOTS + slot; i0 < tn; i0 += RB * U) {
      float kr[U][VEC], vr[U][VEC], qv[U][VEC];
      bool valid[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int i = i0 + u * RB;
        valid[u] = i < tn;
        const int j = s_pos[valid[u] ? i : i0];
        RowVec<T>::load(kb + (size_t)j * kD, kr[u]);
        RowVec<T>::load(vb + (size_t)j * kD, vr[u]);
        const int delta = sr.n - 1 - j;
        if (delta < window) {   // window token: standard RoPE at relative position delta
          const float* cw = cos_win + (size_t)delta * HALF + (d0 & (HALF - 1));
          const float* sw = sin_win + (size_t)delta * HALF + (d0 & (HALF - 1));
#pragma unroll
          for (int v = 0; v < VEC; ++v) qv[u][v] = q_own[v] * cw[v] + q_par[v] * sw[v];
        } else {
#pragma unroll
          for (int v = 0; v < VEC; ++v) qv[u][v] = q_far[v];
        }
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        float dot = 0.f;
#pragma unroll
        for (int v = 0; v < VEC; ++v) dot += qv[u][v] * kr[u][v];
#pragma unroll
        for (int off = 1; off < LPR; off <<= 1) dot += __shfl_xor(dot, off);
        if (valid[u]) {
          const float logit = dot * scale;
          const float mn = fmaxf(m_run, logit);
          const float alpha = __expf(m_run - mn), p = __expf(logit - mn);
          l_run = l_run * alpha + p;
#pragma unroll
          for (int v = 0; v < VEC; ++v) acc[v] = acc[v] * alpha + p * vr[u][v];
          m_run = mn;
        }
      }
    }
  }

  // merge the row slots of a wave, then the waves of the block
#pragma unroll
  for (int off = LPR; off < 64; off <<= 1) {
    const float m2 = __shfl_xor(m_run, off), l2 = __shfl_xor(l_run, off);
    float a2[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) a2[v] = __shfl_xor(acc[v], off);
    merge_state<VEC>(m_run, l_run, acc, m2, l2, a2);
  }
  if (lane < LPR) {
    if (lane == 0) { s_m[wv] = m_run; s_l[wv] = l_run; }
#pragma unroll
    for (int v = 0; v < VEC; ++v) s_acc[wv][d0 + v] = acc[v];
  }
  __syncthreads();
  if (tid < kD) {
    float m = s_m[0], l = s_l[0], a[1] = {s_acc[0][tid]};
    for (int w = 1; w < NWV; ++w) {
      const float a2[1] = {s_acc[w][tid]};
      merge_state<1>(m, l, a, s_m[w], s_l[w], a2);
    }
    if (n_split == 1) {
      store_elem(out + (size_t)bh * kD + tid, l > 0.f ? a[0] / l : 0.f);
    } else {
      float* pp = partial + ((size_t)bh * n_split + split) * (kD + 2);
      pp[tid] = a[0];
      if (tid == 0) { pp[kD] = m; pp[kD + 1] = l; }
    }
  }
}

template <typename T>
__global__ __launch_bounds__(kD) void attn_combine_kernel(const float* __restrict__ partial,
                                                          T* __restrict__ out, int n_split) {
  const int bh = blockIdx.x, d = threadIdx.x;
  const float* pp = partial + (size_t)bh * n_split * (kD + 2);
  float m = -INFINITY;
  for (int s = 0; s < n_split; ++s) m = fmaxf(m, pp[s * (kD + 2) + kD]);
  float l = 0.f, o = 0.f;
  if (m != -INFINITY) {
    for (int s = 0; s < n_split; ++s) {
      const float w = __expf(pp[s * (kD + 2) + kD] - m);
      l += pp[s * (kD + 2) + kD + 1] * w;
      o += pp[s * (kD + 2) + d] * w;
    }
  }
  store_elem(out + (size_t)bh * kD + d, l > 0.f ? o / l : 0.f);
}

template <typename T>
static hipError_t launch_attn_t(const a2ats_dims& d, const AttnPlan& plan, const void* q, const float* q_rot,
                                const void* k_cache, const void* v_cache, const int32_t* topk_idx,
                                const int32_t* topk_count, int top_k, int window, int n_sink,
                                const float* cos_win, const float* sin_win, const int32_t* seq_lens,
                                void* out, void* ws, hipStream_t stream) {
  const int heads = d.batch * d.n_q_heads;
  if (heads == 0) return hipSuccess;
  hipLaunchKernelGGL((attn_partial_kernel<T>), dim3(plan.n_split, heads), dim3(kAttnThreads), 0, stream,
                     (const T*)q, q_rot, (const T*)k_cache, (const T*)v_cache, topk_idx, topk_count,
                     cos_win, sin_win, seq_lens, (T*)out, (float*)ws, d.n_q_heads, d.n_kv_heads,
                     d.ctx_len, d.ctx_stride, top_k, window, n_sink, plan.n_split);
  hipError_t err = hipGetLastError();
  if (err != hipSuccess || plan.n_split == 1) return err;
  hipLaunchKernelGGL((attn_combine_kernel<T>), dim3(heads), dim3(kD), 0, stream, (const float*)ws,
                     (T*)out, plan.n_split);
  return hipGetLastError();
}

hipError_t launch_sparse_attn(const a2ats_dims& d, const void* q, const float* q_rot, const void* k_cache,
                              const void* v_cache, int kv_dtype, const int32_t* topk_idx,
                              const int32_t* topk_count, int top_k, int window, int n_sink,
                              const float* cos_win, const float* sin_win, const int32_t* seq_lens,
                              void* out, void* ws, hipStream_t stream) {
  const AttnPlan plan = make_attn_plan(d, top_k, window, n_sink);
  if (kv_dtype == A2ATS_BF16)
    return launch_attn_t<uint16_t>(d, plan, q, q_rot, k_cache, v_cache, topk_idx, topk_count, top_k,
                                   window, n_sink, cos_win, sin_win, seq_lens, out, ws, stream);
  return launch_attn_t<float>(d, plan, q, q_rot, k_cache, v_cache, topk_idx, topk_count, top_k, window,
                              n_sink, cos_win, sin_win, seq_lens, out, ws, stream);
}

}  // namespace a2ats
