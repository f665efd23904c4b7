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
// triples a second small kernel merges.  With one selection per KV head (the shared variant) the
// far rows are the same for the G heads of a KV head and q~ K^T is a thin matrix product: that case
// (bf16 caches) goes through the matrix cores, see attn_shared_mfma_kernel.
#include <type_traits>

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
__device__ __forceinline__ void attn_partial_body(
    int part, int bh, const T* __restrict__ q, const float* __restrict__ q_rot, const T* __restrict__ k_cache,
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

#define A2ATS_ATTN_ARGS                                                                                \
  const T *__restrict__ q, const float *__restrict__ q_rot, const T *__restrict__ k_cache,               \
      const T *__restrict__ v_cache, const int32_t *__restrict__ topk_idx,                               \
      const int32_t *__restrict__ topk_count, const float *__restrict__ cos_win,                         \
      const float *__restrict__ sin_win, const int32_t *__restrict__ seq_lens,                           \
      float *__restrict__ partial, int Hq, int Hkv, int ctx_len, int64_t ctx_stride, int top_k,          \
      int window, int n_sink, int n_far, int n_win, const int32_t *__restrict__ page_table,              \
      int page_shift, int pages_per_seq
#define A2ATS_ATTN_PASS                                                                                \
  q, q_rot, k_cache, v_cache, topk_idx, topk_count, cos_win, sin_win, seq_lens, partial, Hq, Hkv,        \
      ctx_len, ctx_stride, top_k, window, n_sink, n_far, n_win, page_table, page_shift, pages_per_seq

template <typename T, bool SHARED>
__global__ __launch_bounds__(kAttnThreads) void attn_partial_kernel(A2ATS_ATTN_ARGS) {
  // All workgroups of a (sequence, KV head) run on one XCD, the G heads of a part side by side: the
  // window rows and sinks (per-head selection) or all rows (shared selection) that the G heads have
  // in common come from HBM once and from that XCD's L2 for the others.
  const int G = Hq / Hkv, parts = n_far + n_win;
  int prob, pg;
  xcd_map(blockIdx.x, parts * G, (int)(gridDim.x / (parts * G)), prob, pg);   // prob = b * Hkv + kv
  attn_partial_body<T, SHARED>(pg / G, prob * G + pg % G, A2ATS_ATTN_PASS);
}

// ------------------------------------------------------------------------------------------
// One selection per KV head, bf16 cache: the far rows (sinks + retrieved) of a KV head are the same
// for its G query heads, so q~ K^T is a real (if thin) matrix product: G x 128 times 128 x rows.
// A wave takes 16 rows at a time as the B operand of v_mfma_f32_16x16x32_bf16 (lane = row n +
// 16 * (k / 8): eight consecutive dimensions of one row, straight from the row's memory, no LDS),
// the rotated queries as the A operand (head m in row m, rows >= G zero; the float32 queries are
// split into two bf16 terms so that the logits keep float32-like precision), four k-steps of 32.
// Accumulator register i of lane L holds head 4 * (L / 16) + i, row L % 16.  The softmax
// statistics run over the 16 lanes of a DPP row; P V stays on the vector ALU with the
// probabilities broadcast through scalar registers: every lane owns two output dimensions and a
// value row is read with one coalesced 4-byte load per lane.  Each row comes from HBM once for all
// G heads.  GP: G padded to 4 or 8.
typedef __attribute__((ext_vector_type(8))) __bf16 attn_bf16x8;
typedef __attribute__((ext_vector_type(4))) float attn_f32x4;

__device__ __forceinline__ float row16_max(float v) {
  v = fmaxf(v, __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0xB1, 0xf, 0xf, false)));
  v = fmaxf(v, __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x4E, 0xf, 0xf, false)));
  v = fmaxf(v, __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x141, 0xf, 0xf, false)));
  v = fmaxf(v, __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x140, 0xf, 0xf, false)));
  return v;
}
__device__ __forceinline__ float lane_value(float v, int src_lane) {   // src_lane: a compile-time constant
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), src_lane));
}

template <int GP>
__device__ __forceinline__ void attn_far_shared_mfma_body(
    int prob, int part, const float* __restrict__ q_rot, const uint16_t* __restrict__ k_cache,
    const uint16_t* __restrict__ v_cache, const int32_t* __restrict__ topk_idx,
    const int32_t* __restrict__ topk_count, const int32_t* __restrict__ seq_lens, float* __restrict__ partial,
    int Hq, int Hkv, int ctx_len, int64_t ctx_stride, int top_k, int window, int n_sink, int n_far, int n_win,
    const int32_t* __restrict__ page_table, int page_shift, int pages_per_seq) {
  constexpr int NWV = kAttnThreads / 64;
  __shared__ uint32_t s_row[kAttnTile];
  __shared__ float s_m[NWV][GP], s_l[NWV][GP], s_o[NWV][GP][kD];

  const int G = Hq / Hkv;
  const int b = prob / Hkv, kv = prob % Hkv;   // prob = b * Hkv + kv
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, n = lane & 15, kg = lane >> 4;
  const SeqRange sr = seq_range(ctx_len, seq_lens, b, window, n_sink, top_k);
  const int cnt = max(0, min(min(topk_count[prob], top_k), sr.ncand));
  const int n_rows = sr.sink_end + cnt;
  const int n_mine = n_rows > part ? (n_rows - part + n_far - 1) / n_far : 0;
  const size_t seq_base = page_table ? 0 : ((size_t)b * Hkv + kv) * ctx_stride * kD;
  const uint16_t* kb = k_cache + seq_base;
  const uint16_t* vb = v_cache + seq_base;
  const int32_t* pages = page_table ? page_table + (size_t)b * pages_per_seq : nullptr;
  const int32_t* idx = topk_idx + (size_t)prob * top_k;
  const float scale = 0.08838834764831845f;   // 1/sqrt(128)

  // A operand: head n of the KV head, dimensions 32 s + 8 kg .. + 8, as hi + lo bf16 (rows >= G: zero).
  // Eight 16-byte loads per lane, all in flight together; hi is the float truncated to bf16 and lo
  // the (exactly representable) rest rounded down to bf16, packed with integer operations.  (A first
  // version filled the operand vectors element by element from 32 scalar loads: 6.5 us before the
  // first row was requested.)
  attn_bf16x8 a_hi[4], a_lo[4];
  {
    const float4* qh = (const float4*)(q_rot + ((size_t)b * Hq + (size_t)kv * G + (n < G ? n : 0)) * kD + kg * 8);
    float4 qv[8];
#pragma unroll
    for (int s_ = 0; s_ < 4; ++s_) {
      qv[2 * s_] = qh[s_ * 8];
      qv[2 * s_ + 1] = qh[s_ * 8 + 1];
    }
    const float keep = n < G ? 1.f : 0.f;
#pragma unroll
    for (int s_ = 0; s_ < 4; ++s_) {
      const float x[8] = {qv[2 * s_].x, qv[2 * s_].y, qv[2 * s_].z, qv[2 * s_].w,
                          qv[2 * s_ + 1].x, qv[2 * s_ + 1].y, qv[2 * s_ + 1].z, qv[2 * s_ + 1].w};
      uint32_t hw[4], lw[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float x0 = x[2 * e] * keep, x1 = x[2 * e + 1] * keep;
        const uint32_t h0 = __float_as_uint(x0) & 0xffff0000u, h1 = __float_as_uint(x1) & 0xffff0000u;
        const float r0 = x0 - __uint_as_float(h0), r1 = x1 - __uint_as_float(h1);   // exact
        hw[e] = (h0 >> 16) | h1;
        lw[e] = (__float_as_uint(r0) >> 16) | (__float_as_uint(r1) & 0xffff0000u);
      }
      a_hi[s_] = __builtin_bit_cast(attn_bf16x8, make_uint4(hw[0], hw[1], hw[2], hw[3]));
      a_lo[s_] = __builtin_bit_cast(attn_bf16x8, make_uint4(lw[0], lw[1], lw[2], lw[3]));
    }
  }

  // running state of head 4 kg + i (identical in the 16 lanes of a lane group) and this lane's two
  // output dimensions (2 lane, 2 lane + 1) of every head
  float m_run[4], l_run[4], o[GP][2];
#pragma unroll
  for (int i = 0; i < 4; ++i) { m_run[i] = -INFINITY; l_run[i] = 0.f; }
#pragma unroll
  for (int g = 0; g < GP; ++g) { o[g][0] = 0.f; o[g][1] = 0.f; }

  for (int tb = 0; tb < n_mine; tb += kAttnTile) {
    const int tn = min(kAttnTile, n_mine - tb);
    __syncthreads();
    for (int i = tid; i < tn; i += kAttnThreads) {
      const int t = part + (tb + i) * n_far;
      int j = t < sr.sink_end ? t : idx[t - sr.sink_end];
      j = min(max(j, 0), sr.n - 1);   // a bad caller index must not leave the cache
      s_row[i] = pages ? (((uint32_t)pages[j >> page_shift] * (uint32_t)Hkv + (uint32_t)kv) << page_shift) +
                             (uint32_t)(j & ((1 << page_shift) - 1))
                       : (uint32_t)j;
    }
    __syncthreads();

    // Tiles of 16 rows, dealt to the waves in turn; the next tile's rows are requested
    // (unconditionally, tile index clamped) before the current one is used: two register sets.
    const int n_tiles = (tn + 15) >> 4;
    uint4 kA[4], kB[4];
    uint32_t vA[16], vB[16];
    auto load_tile = [&](int tile, uint4 (&kr)[4], uint32_t (&vr)[16]) {
      const int t0 = min(tile, n_tiles - 1) << 4;
      const uint32_t row = s_row[min(t0 + n, tn - 1)];
      const uint16_t* kp = kb + (size_t)row * kD + kg * 8;
#pragma unroll
      for (int s_ = 0; s_ < 4; ++s_) kr[s_] = *(const uint4*)(kp + s_ * 32);
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const uint32_t rr = s_row[min(t0 + r, tn - 1)];   // (one address for the wave: an LDS broadcast)
        vr[r] = *(const uint32_t*)(vb + (size_t)rr * kD + 2 * lane);
      }
    };
    auto use_tile = [&](int tile, const uint4 (&kr)[4], const uint32_t (&vr)[16]) {
      const int t0 = tile << 4;
      attn_f32x4 sacc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int s_ = 0; s_ < 4; ++s_) {
        const attn_bf16x8 bk = __builtin_bit_cast(attn_bf16x8, kr[s_]);
        sacc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a_hi[s_], bk, sacc, 0, 0, 0);
        sacc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a_lo[s_], bk, sacc, 0, 0, 0);
      }
      const bool valid = t0 + n < tn;
      float pr[4], alpha[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float logit = valid ? sacc[i] * scale : -INFINITY;
        const float mn = fmaxf(m_run[i], row16_max(logit));   // finite: a tile has at least one valid row
        alpha[i] = __expf(m_run[i] - mn);
        pr[i] = __expf(logit - mn);
        l_run[i] = l_run[i] * alpha[i] + row16_sum(pr[i]);
        m_run[i] = mn;
      }
      float v0[16], v1[16];
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        v0[r] = __uint_as_float(vr[r] << 16);
        v1[r] = __uint_as_float(vr[r] & 0xffff0000u);
      }
#pragma unroll
      for (int g = 0; g < GP; ++g) {
        const int i = g & 3, src = 16 * (g >> 2);   // head g: register i of lane group g / 4
        const float al = lane_value(alpha[i], src);
        float o0 = o[g][0] * al, o1 = o[g][1] * al;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float pv = lane_value(pr[i], src + r);
          o0 += pv * v0[r];
          o1 += pv * v1[r];
        }
        o[g][0] = o0;
        o[g][1] = o1;
      }
    };
    load_tile(wv, kA, vA);
#pragma unroll 1
    for (int tile = wv; tile < n_tiles; tile += 2 * NWV) {
      load_tile(tile + NWV, kB, vB);
      use_tile(tile, kA, vA);
      load_tile(tile + 2 * NWV, kA, vA);
      if (tile + NWV < n_tiles) use_tile(tile + NWV, kB, vB);
    }
  }

  // merge the waves of the block, one thread per output dimension, head by head
  if (n == 0 && kg < GP / 4) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      s_m[wv][4 * kg + i] = m_run[i];
      s_l[wv][4 * kg + i] = l_run[i];
    }
  }
#pragma unroll
  for (int g = 0; g < GP; ++g) {
    s_o[wv][g][2 * lane] = o[g][0];
    s_o[wv][g][2 * lane + 1] = o[g][1];
  }
  __syncthreads();
  if (tid < kD) {
    for (int g = 0; g < G; ++g) {
      float m = s_m[0][g], l = s_l[0][g], a[1] = {s_o[0][g][tid]};
      for (int w = 1; w < NWV; ++w) {
        const float a2[1] = {s_o[w][g][tid]};
        merge_state<1>(m, l, a, s_m[w][g], s_l[w][g], a2);
      }
      const size_t bh = (size_t)b * Hq + (size_t)kv * G + g;
      float* pp = partial + (bh * (n_far + n_win) + part) * (kD + 2);
      pp[tid] = a[0];
      if (tid == 0) { pp[kD] = m; pp[kD + 1] = l; }
    }
  }
}

// The launch of the shared selection: the first n_far workgroups of every (sequence, KV head) take the
// far rows on the matrix cores for all G heads; after them come, per query head, the n_win workgroups
// of the window rows (a rotation per row: the per-head vector-ALU path), mapped so that the G heads of a
// KV head read the same rows side by side on one XCD.
template <int GP>
__global__ __launch_bounds__(kAttnThreads) void attn_shared_mfma_kernel(
    const uint16_t* __restrict__ q, const float* __restrict__ q_rot, const uint16_t* __restrict__ k_cache,
    const uint16_t* __restrict__ v_cache, const int32_t* __restrict__ topk_idx,
    const int32_t* __restrict__ topk_count, const float* __restrict__ cos_win,
    const float* __restrict__ sin_win, const int32_t* __restrict__ seq_lens, float* __restrict__ partial,
    int Hq, int Hkv, int ctx_len, int64_t ctx_stride, int top_k, int window, int n_sink, int n_far, int n_win,
    const int32_t* __restrict__ page_table, int page_shift, int pages_per_seq, int problems) {
  const int far_blocks = n_far * problems;
  if ((int)blockIdx.x < far_blocks) {   // (uniform over the workgroup)
    int prob, part;
    xcd_map(blockIdx.x, n_far, problems, prob, part);
    attn_far_shared_mfma_body<GP>(prob, part, q_rot, k_cache, v_cache, topk_idx, topk_count, seq_lens, partial, Hq,
                                  Hkv, ctx_len, ctx_stride, top_k, window, n_sink, n_far, n_win, page_table,
                                  page_shift, pages_per_seq);
  } else {
    const int G = Hq / Hkv;
    int prob, pg;
    xcd_map((int)blockIdx.x - far_blocks, n_win * G, problems, prob, pg);
    attn_partial_body<uint16_t, true>(n_far + pg / G, prob * G + pg % G, q, q_rot, k_cache, v_cache, topk_idx,
                                      topk_count, cos_win, sin_win, seq_lens, partial, Hq, Hkv, ctx_len, ctx_stride,
                                      top_k, window, n_sink, n_far, n_win, page_table, page_shift, pages_per_seq);
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
  const int G = d.n_q_heads / d.n_kv_heads;
  if (shared && std::is_same<T, uint16_t>::value && G <= 8) {
    // bf16 cache: far rows on the matrix cores once per KV head, window rows per head, one launch
    const int problems = d.batch * d.n_kv_heads;
    const dim3 grid(plan.n_far * problems + plan.n_win * heads);
    if (G <= 4)
      hipLaunchKernelGGL((attn_shared_mfma_kernel<4>), grid, dim3(kAttnThreads), 0, stream, (const uint16_t*)q, q_rot,
                         (const uint16_t*)k_cache, (const uint16_t*)v_cache, topk_idx, topk_count, cos_win, sin_win,
                         seq_lens, (float*)ws, d.n_q_heads, d.n_kv_heads, d.ctx_len, d.ctx_stride, top_k, window,
                         n_sink, plan.n_far, plan.n_win, page_table, page_shift, pages_per_seq, problems);
    else
      hipLaunchKernelGGL((attn_shared_mfma_kernel<8>), grid, dim3(kAttnThreads), 0, stream, (const uint16_t*)q, q_rot,
                         (const uint16_t*)k_cache, (const uint16_t*)v_cache, topk_idx, topk_count, cos_win, sin_win,
                         seq_lens, (float*)ws, d.n_q_heads, d.n_kv_heads, d.ctx_len, d.ctx_stride, top_k, window,
                         n_sink, plan.n_far, plan.n_win, page_table, page_shift, pages_per_seq, problems);
  } else if (shared)
    hipLaunchKernelGGL((attn_partial_kernel<T, true>), dim3(parts * heads), dim3(kAttnThreads), 0, stream,
                       (const T*)q, q_rot, (const T*)k_cache, (const T*)v_cache, topk_idx, topk_count,
                       cos_win, sin_win, seq_lens, (float*)ws, d.n_q_heads, d.n_kv_heads, d.ctx_len,
                       d.ctx_stride, top_k, window, n_sink, plan.n_far, plan.n_win, page_table, page_shift,
                       pages_per_seq);
  else
    hipLaunchKernelGGL((attn_partial_kernel<T, false>), dim3(parts * heads), dim3(kAttnThreads), 0, stream,
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
