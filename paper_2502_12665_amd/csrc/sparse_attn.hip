// Step 4 of a decode step: exact attention over sinks U top-K U window under WRoPE
// (section 2.1 eq. "output state" restricted to the attended set; section 4.1 eq. "WRoPE").
//
// The phase is a random-row gather from HBM: per query head about K + w key rows and as many
// value rows of 256 B (bf16) or 512 B (float32) each, 2 flop per byte fetched.  Every query
// head has its own retrieved set, so the "matrix" on the query side has one row; the
// products are therefore done on the vector ALU and all effort goes into keeping many row
// loads in flight: a row is read by 16 (bf16) or 32 (float32) lanes with one 16-byte load
// each, a wave works on 4 (2) rows at a time with a second set of rows already requested, and
// the rows of one head are split over several workgroups whose partial (max, sum, accumulator)
// triples a second small kernel merges.
#include "common.hpp"
#include "internal.hpp"

namespace a2ats {

constexpr int kAttnThreads = 256;
constexpr int kAttnTile = 512;   // positions staged in LDS at a time
constexpr int kD = 128;

AttnPlan make_attn_plan(const a2ats_dims& d, int top_k, int window, int n_sink) {
  // Workgroups of a head: n_far share the sinks and the retrieved rows, n_win the window rows
  // (which need the per-row rotation and are kept apart so that the common path has no branch).
  AttnPlan p;
  const long heads = (long)d.batch * d.n_q_heads;
  long far_rows = (long)n_sink + top_k;
  if (far_rows > d.ctx_len) far_rows = d.ctx_len;
  long nf = heads > 0 ? (1024 + heads - 1) / heads : 1;
  const long by_rows = far_rows / 64 > 1 ? far_rows / 64 : 1;
  if (nf > by_rows) nf = by_rows;
  if (nf > 32) nf = 32;
  if (nf < 1) nf = 1;
  long nw = ((long)window + 127) / 128;
  if (nw > 8) nw = 8;
  if (nw < 1) nw = 1;
  p.n_far = (int)nf;
  p.n_win = (int)nw;
  p.bytes = (size_t)heads * (nf + nw) * (kD + 2) * sizeof(float);
  return p;
}

// A lane's 16-byte piece of a row, kept as loaded (so that rows in flight cost four registers
// each) and widened to float only when it is used.
template <typename T> struct RowVec;
template <> struct RowVec<float> {
  static constexpr int LPR = 32, VEC = 4;
  static __device__ __forceinline__ uint4 load(const float* p) { return *(const uint4*)p; }
  static __device__ __forceinline__ void widen(const uint4& v, float (&o)[4]) {
    o[0] = __uint_as_float(v.x); o[1] = __uint_as_float(v.y);
    o[2] = __uint_as_float(v.z); o[3] = __uint_as_float(v.w);
  }
};
template <> struct RowVec<uint16_t> {
  static constexpr int LPR = 16, VEC = 8;
  static __device__ __forceinline__ uint4 load(const uint16_t* p) { return *(const uint4*)p; }
  static __device__ __forceinline__ void widen(const uint4& v, float (&o)[8]) {
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

// Sum over the 16 lanes of a DPP row, result in every lane: two swaps inside quads, then the mirror
// images within 8 and within 16 lanes.  (A __shfl_xor is a round trip through the LDS crossbar; four
// of them in a chain per attended row were the longest dependency of the kernel.)  The 16 lanes must
// be all active or all inactive.
__device__ __forceinline__ float row16_sum(float v) {
  v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0xB1, 0xf, 0xf, false));    // quad_perm [1,0,3,2]
  v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x4E, 0xf, 0xf, false));    // quad_perm [2,3,0,1]
  v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x141, 0xf, 0xf, false));   // row_half_mirror
  v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x140, 0xf, 0xf, false));   // row_mirror
  return v;
}

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

// SHARED: topk_idx / topk_count are per KV head and the G query heads of a KV head attend the same
// rows.  The grid is then one-dimensional and mapped so that the G workgroups that read the same
// rows (same KV head, same part) run next to each other on one XCD: the rows come from HBM once
// and from that XCD's L2 for the other G - 1 heads.
template <typename T, bool SHARED>
__global__ __launch_bounds__(kAttnThreads) void attn_partial_kernel(
    const T* __restrict__ q, const float* __restrict__ q_rot, const T* __restrict__ k_cache,
    const T* __restrict__ v_cache, const int32_t* __restrict__ topk_idx,
    const int32_t* __restrict__ topk_count, const float* __restrict__ cos_win,
    const float* __restrict__ sin_win, const int32_t* __restrict__ seq_lens,
    float* __restrict__ partial, int Hq, int Hkv, int ctx_len, int64_t ctx_stride, int top_k,
    int window, int n_sink, int n_far, int n_win, const int32_t* __restrict__ page_table, int page_shift,
    int pages_per_seq) {
  // page_table != NULL: k_cache / v_cache are pools of pages [page][Hkv][2^page_shift][D] and token j of
  // sequence b lives in page page_table[b][j >> page_shift]; else row j of [B][Hkv][ctx_stride][D].
  constexpr int LPR = RowVec<T>::LPR, VEC = RowVec<T>::VEC;
  constexpr int SLOTS = 64 / LPR;            // rows a wave reads at once
  constexpr int NWV = kAttnThreads / 64;
  constexpr int RB = NWV * SLOTS;            // rows per block step
  constexpr int HALF = kD / 2;
  __shared__ int32_t s_pos[kAttnTile];     // token positions of the staged rows
  __shared__ uint32_t s_row[kAttnTile];    // their row numbers in the cache (or pool)
  __shared__ float s_m[NWV], s_l[NWV], s_acc[NWV][kD];

  const int G = Hq / Hkv;
  int part, bh;
  if (SHARED) {
    const int parts = n_far + n_win;
    int prob, pg;
    xcd_map(blockIdx.x, parts * G, (int)(gridDim.x / (parts * G)), prob, pg);
    part = pg / G;
    bh = prob * G + pg % G;   // prob = b * Hkv + kv
  } else {
    part = blockIdx.x;
    bh = blockIdx.y;
  }
  const int b = bh / Hq, h = bh % Hq, kv = h / G;
  const int ih = SHARED ? b * Hkv + kv : bh;   // whose selection this head attends
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, slot = lane / LPR, sub = lane % LPR;
  const SeqRange sr = seq_range(ctx_len, seq_lens, b, window, n_sink, top_k);
  const int cnt = max(0, min(min(topk_count[ih], top_k), sr.ncand));
  // Far rows (sinks, then the retrieved rows) are dealt out round-robin to the first n_far
  // workgroups of the head, window rows to the other n_win.
  const bool win_part = part >= n_far;
  const int n_rows = win_part ? sr.n - sr.win_start : sr.sink_end + cnt;
  const int stride = win_part ? n_win : n_far, first = win_part ? part - n_far : part;
  const int n_mine = n_rows > first ? (n_rows - first + stride - 1) / stride : 0;

  const int d0 = sub * VEC;
  const float scale = 0.08838834764831845f;   // 1/sqrt(128)
  const size_t seq_base = page_table ? 0 : ((size_t)b * Hkv + kv) * ctx_stride * kD;
  const T* kb = k_cache + seq_base + d0;
  const T* vb = v_cache + seq_base + d0;
  const int32_t* pages = page_table ? page_table + (size_t)b * pages_per_seq : nullptr;
  const int32_t* idx = topk_idx + (size_t)ih * top_k;
  const size_t qb = (size_t)bh * kD;

  float m_run = -INFINITY, l_run = 0.f, acc[VEC];
#pragma unroll
  for (int v = 0; v < VEC; ++v) acc[v] = 0.f;

  // One row's contribution, given this lane's part of q . k
  auto absorb = [&](float dot, const uint4& vraw) {
    dot = row16_sum(dot);
    if (LPR == 32) dot += __shfl_xor(dot, 16);   // a float32 row spans two DPP rows
    float vr[VEC];
    RowVec<T>::widen(vraw, vr);
    const float logit = dot * scale;
    const float mn = fmaxf(m_run, logit);
    const float alpha = __expf(m_run - mn), pr = __expf(logit - mn);
    l_run = l_run * alpha + pr;
#pragma unroll
    for (int v = 0; v < VEC; ++v) acc[v] = acc[v] * alpha + pr * vr[v];
    m_run = mn;
  };

  for (int tb = 0; tb < n_mine; tb += kAttnTile) {
    const int tn = min(kAttnTile, n_mine - tb);
    __syncthreads();
    for (int i = tid; i < tn; i += kAttnThreads) {
      const int t = first + (tb + i) * stride;
      int j;
      if (win_part) j = sr.win_start + t;
      else j = t < sr.sink_end ? t : idx[t - sr.sink_end];
      j = min(max(j, 0), sr.n - 1);   // a bad caller index must not leave the cache
      s_pos[i] = j;
      s_row[i] = pages ? (((uint32_t)pages[j >> page_shift] * (uint32_t)Hkv + (uint32_t)kv) << page_shift) +
                             (uint32_t)(j & ((1 << page_shift) - 1))
                       : (uint32_t)j;
    }
    __syncthreads();

    if (!win_part) {
      // Far rows: logit = q~ . k.  Two register sets of U rows are used alternately: the loads of
      // one are issued (unconditionally, row index clamped) before the other is consumed, so a
      // wave always has 2 U key and value rows in flight.
      constexpr int U = 2;
      constexpr int STEP = RB * U;
      float q_far[VEC];
#pragma unroll
      for (int v = 0; v < VEC; ++v) q_far[v] = q_rot[qb + d0 + v];
      uint4 ka[U], va[U], kc[U], vc[U];
      auto load_set = [&](int i0, uint4 (&kr)[U], uint4 (&vr)[U]) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const uint32_t row = s_row[min(i0 + u * RB, tn - 1)];
          kr[u] = RowVec<T>::load(kb + (size_t)row * kD);
          vr[u] = RowVec<T>::load(vb + (size_t)row * kD);
        }
      };
      auto use_set = [&](int i0, const uint4 (&kr)[U], const uint4 (&vr)[U]) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
          float kf[VEC];
          RowVec<T>::widen(kr[u], kf);
          float dot = 0.f;
#pragma unroll
          for (int v = 0; v < VEC; ++v) dot += q_far[v] * kf[v];
          if (i0 + u * RB < tn) absorb(dot, vr[u]);
        }
      };
      const int lane_row = wv * SLOTS + slot;
      load_set(lane_row, ka, va);
#pragma unroll 1
      for (int base = 0; base < tn; base += 2 * STEP) {
        load_set(base + STEP + lane_row, kc, vc);
        use_set(base + lane_row, ka, va);
        load_set(base + 2 * STEP + lane_row, ka, va);
        use_set(base + STEP + lane_row, kc, vc);
      }
    } else {
      // Window rows: logit = (q R_delta) . k with the standard rotation at the relative position
      // delta = n - 1 - j, built from the cos/sin tables of the row.
      constexpr int U = 2;
      const bool low_half = d0 < HALF;
      const int dp = low_half ? d0 + HALF : d0 - HALF;
      const float sgn = low_half ? -1.f : 1.f;
      float q_own[VEC], q_par[VEC];
#pragma unroll
      for (int v = 0; v < VEC; ++v) {
        q_own[v] = load_elem(q + qb + d0 + v);
        q_par[v] = load_elem(q + qb + dp + v) * sgn;
      }
      for (int i0 = wv * SLOTS + slot; i0 < tn; i0 += RB * U) {
        uint4 kr[U], vr[U];
        float cw[U][VEC], sw[U][VEC];
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const int j = s_pos[min(i0 + u * RB, tn - 1)];
          const uint32_t row = s_row[min(i0 + u * RB, tn - 1)];
          kr[u] = RowVec<T>::load(kb + (size_t)row * kD);
          vr[u] = RowVec<T>::load(vb + (size_t)row * kD);
          const int delta = min(max(sr.n - 1 - j, 0), window - 1);
          const float* cp = cos_win + (size_t)delta * HALF + (d0 & (HALF - 1));
          const float* sp = sin_win + (size_t)delta * HALF + (d0 & (HALF - 1));
#pragma unroll
          for (int v = 0; v < VEC; ++v) {
            cw[u][v] = cp[v];
            sw[u][v] = sp[v];
          }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
          float kf[VEC];
          RowVec<T>::widen(kr[u], kf);
          float dot = 0.f;
#pragma unroll
          for (int v = 0; v < VEC; ++v) dot += (q_own[v] * cw[u][v] + q_par[v] * sw[u][v]) * kf[v];
          if (i0 + u * RB < tn) absorb(dot, vr[u]);
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
    float* pp = partial + ((size_t)bh * (n_far + n_win) + part) * (kD + 2);
    pp[tid] = a[0];
    if (tid == 0) { pp[kD] = m; pp[kD + 1] = l; }
  }
}

// Merge the partial states of a head: 4 groups of 128 threads (one thread per output dimension)
// each fold every fourth state into a running one -- four states' loads are issued together, so a
// head with up to 16 workgroups costs one load latency -- then the four are folded through LDS.
constexpr int kCombineGroups = 4;
template <typename T>
__global__ __launch_bounds__(kCombineGroups* kD) void attn_combine_kernel(const float* __restrict__ partial,
                                                                         T* __restrict__ out, int n_states) {
  __shared__ float s_m[kCombineGroups], s_l[kCombineGroups], s_o[kCombineGroups][kD];
  const int bh = blockIdx.x, d = threadIdx.x % kD, g = threadIdx.x / kD;
  const float* pp = partial + (size_t)bh * n_states * (kD + 2);
  float m = -INFINITY, l = 0.f, o = 0.f;
  constexpr int UN = 4;
  for (int s0 = g; s0 < n_states; s0 += kCombineGroups * UN) {
    float pm[UN], pl[UN], po[UN];
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      const int s = min(s0 + u * kCombineGroups, n_states - 1);
      pm[u] = pp[(size_t)s * (kD + 2) + kD];
      pl[u] = pp[(size_t)s * (kD + 2) + kD + 1];
      po[u] = pp[(size_t)s * (kD + 2) + d];
    }
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      if (s0 + u * kCombineGroups < n_states && pm[u] != -INFINITY) {
        const float mn = fmaxf(m, pm[u]);
        const float a = __expf(m - mn), c = __expf(pm[u] - mn);
        l = l * a + pl[u] * c;
        o = o * a + po[u] * c;
        m = mn;
      }
    }
  }
  if (d == 0) { s_m[g] = m; s_l[g] = l; }
  s_o[g][d] = o;
  __syncthreads();
  if (g == 0) {
    float mm = s_m[0];
#pragma unroll
    for (int i = 1; i < kCombineGroups; ++i) mm = fmaxf(mm, s_m[i]);
    float lt = 0.f, ot = 0.f;
    if (mm != -INFINITY) {
#pragma unroll
      for (int i = 0; i < kCombineGroups; ++i) {
        const float w = __expf(s_m[i] - mm);   // exp(-inf) = 0 for an empty group
        lt += s_l[i] * w;
        ot += s_o[i][d] * w;
      }
    }
    store_elem(out + (size_t)bh * kD + d, lt > 0.f ? ot / lt : 0.f);
  }
}

template <typename T>
static hipError_t launch_attn_t(const a2ats_dims& d, const AttnPlan& plan, const void* q, const float* q_rot,
                                const void* k_cache, const void* v_cache, const int32_t* topk_idx,
                                const int32_t* topk_count, int top_k, int window, int n_sink,
                                const float* cos_win, const float* sin_win, const int32_t* seq_lens,
                                void* out, void* ws, bool shared, const int32_t* page_table, int page_shift,
                                hipStream_t stream) {
  const int heads = d.batch * d.n_q_heads;
  const int pages_per_seq = page_table ? (int)((d.ctx_stride + (1 << page_shift) - 1) >> page_shift) : 0;
  if (heads == 0) return hipSuccess;
  const int parts = plan.n_far + plan.n_win;
  if (shared)
    hipLaunchKernelGGL((attn_partial_kernel<T, true>), dim3(parts * heads), dim3(kAttnThreads), 0, stream,
                       (const T*)q, q_rot, (const T*)k_cache, (const T*)v_cache, topk_idx, topk_count,
                       cos_win, sin_win, seq_lens, (float*)ws, d.n_q_heads, d.n_kv_heads, d.ctx_len,
                       d.ctx_stride, top_k, window, n_sink, plan.n_far, plan.n_win, page_table, page_shift,
                       pages_per_seq);
  else
    hipLaunchKernelGGL((attn_partial_kernel<T, false>), dim3(parts, heads), dim3(kAttnThreads), 0, stream,
                       (const T*)q, q_rot, (const T*)k_cache, (const T*)v_cache, topk_idx, topk_count,
                       cos_win, sin_win, seq_lens, (float*)ws, d.n_q_heads, d.n_kv_heads, d.ctx_len,
                       d.ctx_stride, top_k, window, n_sink, plan.n_far, plan.n_win, page_table, page_shift,
                       pages_per_seq);
  hipError_t err = hipGetLastError();
  if (err != hipSuccess) return err;
  hipLaunchKernelGGL((attn_combine_kernel<T>), dim3(heads), dim3(kCombineGroups * kD), 0, stream,
                     (const float*)ws, (T*)out, parts);
  return hipGetLastError();
}

hipError_t launch_sparse_attn(const a2ats_dims& d, const void* q, const float* q_rot, const void* k_cache,
                              const void* v_cache, int kv_dtype, const int32_t* topk_idx,
                              const int32_t* topk_count, int top_k, int window, int n_sink,
                              const float* cos_win, const float* sin_win, const int32_t* seq_lens,
                              void* out, void* ws, bool shared, const int32_t* page_table, int page_shift,
                              hipStream_t stream) {
  const AttnPlan plan = make_attn_plan(d, top_k, window, n_sink);
  if (kv_dtype == A2ATS_BF16)
    return launch_attn_t<uint16_t>(d, plan, q, q_rot, k_cache, v_cache, topk_idx, topk_count, top_k,
                                   window, n_sink, cos_win, sin_win, seq_lens, out, ws, shared, page_table, page_shift,
                                   stream);
  return launch_attn_t<float>(d, plan, q, q_rot, k_cache, v_cache, topk_idx, topk_count, top_k, window,
                              n_sink, cos_win, sin_win, seq_lens, out, ws, shared, page_table, page_shift, stream);
}

}  // namespace a2ats
