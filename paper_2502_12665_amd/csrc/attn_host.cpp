// Selective attention on the host CPU for a key/value cache that lives in host memory: the
// placement of section 4.3 (the GPU scores and selects, the CPU attends over the retrieved tokens
// next to the cache, only indices, the query and the output cross the bus).  Same function as
// a2ats_sparse_attn: exact attention over sinks U top-K U window under WRoPE (section 2.1 eq.
// "output state" restricted to the attended set; section 4.1 eq. "WRoPE").
//
// Host code only (no HIP): one query head per OpenMP task, rows processed in blocks of 32 with an
// online softmax per block, key and value rows prefetched a block ahead (the phase is a random-row
// gather from DRAM; the arithmetic is 2 flop per byte), AVX2 + FMA inner loops chosen at run time
// with a scalar form for other CPUs.  float32 accumulation, like the GPU kernel.
#include <math.h>
#include <stdint.h>
#include <string.h>

#include <algorithm>
#include <vector>

#if defined(__x86_64__)
#include <immintrin.h>
#endif
#include <omp.h>

#include "a2ats.h"

namespace {

constexpr int kD = 128;
constexpr int kBlock = 32;

inline float bf16_to_f32(uint16_t h) {
  uint32_t u = (uint32_t)h << 16;
  float f;
  memcpy(&f, &u, 4);
  return f;
}
inline uint16_t f32_to_bf16(float f) {   // round to nearest even; NaN stays NaN
  uint32_t u;
  memcpy(&u, &f, 4);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

// ---- row primitives: dot(q, row) and acc += p * row, for bf16 and float32 rows -------------------
struct ScalarOps {
  static float dot(const float* q, const uint16_t* r) {
    float s = 0.f;
    for (int i = 0; i < kD; ++i) s += q[i] * bf16_to_f32(r[i]);
    return s;
  }
  static float dot(const float* q, const float* r) {
    float s = 0.f;
    for (int i = 0; i < kD; ++i) s += q[i] * r[i];
    return s;
  }
  static void axpy(float* acc, float p, const uint16_t* r) {
    for (int i = 0; i < kD; ++i) acc[i] += p * bf16_to_f32(r[i]);
  }
  static void axpy(float* acc, float p, const float* r) {
    for (int i = 0; i < kD; ++i) acc[i] += p * r[i];
  }
  static void scale(float* acc, float a) {
    for (int i = 0; i < kD; ++i) acc[i] *= a;
  }
};

#if defined(__x86_64__)
#define A2ATS_AVX2 __attribute__((target("avx2,fma")))
struct Avx2Ops {
  A2ATS_AVX2 static __m256 widen(const uint16_t* p) {
    return _mm256_castsi256_ps(_mm256_slli_epi32(_mm256_cvtepu16_epi32(_mm_loadu_si128((const __m128i*)p)), 16));
  }
  A2ATS_AVX2 static float hsum(__m256 v) {
    __m128 s = _mm_add_ps(_mm256_castps256_ps128(v), _mm256_extractf128_ps(v, 1));
    s = _mm_add_ps(s, _mm_movehl_ps(s, s));
    s = _mm_add_ss(s, _mm_shuffle_ps(s, s, 1));
    return _mm_cvtss_f32(s);
  }
  A2ATS_AVX2 static float dot(const float* q, const uint16_t* r) {
    __m256 a0 = _mm256_setzero_ps(), a1 = _mm256_setzero_ps();
    for (int i = 0; i < kD; i += 16) {
      a0 = _mm256_fmadd_ps(_mm256_loadu_ps(q + i), widen(r + i), a0);
      a1 = _mm256_fmadd_ps(_mm256_loadu_ps(q + i + 8), widen(r + i + 8), a1);
    }
    return hsum(_mm256_add_ps(a0, a1));
  }
  A2ATS_AVX2 static float dot(const float* q, const float* r) {
    __m256 a0 = _mm256_setzero_ps(), a1 = _mm256_setzero_ps();
    for (int i = 0; i < kD; i += 16) {
      a0 = _mm256_fmadd_ps(_mm256_loadu_ps(q + i), _mm256_loadu_ps(r + i), a0);
      a1 = _mm256_fmadd_ps(_mm256_loadu_ps(q + i + 8), _mm256_loadu_ps(r + i + 8), a1);
    }
    return hsum(_mm256_add_ps(a0, a1));
  }
  A2ATS_AVX2 static void axpy(float* acc, float p, const uint16_t* r) {
    const __m256 pv = _mm256_set1_ps(p);
    for (int i = 0; i < kD; i += 8) _mm256_storeu_ps(acc + i, _mm256_fmadd_ps(pv, widen(r + i), _mm256_loadu_ps(acc + i)));
  }
  A2ATS_AVX2 static void axpy(float* acc, float p, const float* r) {
    const __m256 pv = _mm256_set1_ps(p);
    for (int i = 0; i < kD; i += 8)
      _mm256_storeu_ps(acc + i, _mm256_fmadd_ps(pv, _mm256_loadu_ps(r + i), _mm256_loadu_ps(acc + i)));
  }
  A2ATS_AVX2 static void scale(float* acc, float a) {
    const __m256 av = _mm256_set1_ps(a);
    for (int i = 0; i < kD; i += 8) _mm256_storeu_ps(acc + i, _mm256_mul_ps(av, _mm256_loadu_ps(acc + i)));
  }
};
#endif

inline void prefetch_row(const void* p, size_t bytes) {
#if defined(__x86_64__)
  for (size_t o = 0; o < bytes; o += 64) _mm_prefetch((const char*)p + o, _MM_HINT_T0);
#else
  (void)p;
  (void)bytes;
#endif
}

struct Geometry {
  int n, win_start, sink_end, ncand;
};
inline Geometry geometry(int ctx_len, const int32_t* seq_lens, int b, int window, int n_sink) {
  Geometry g;
  g.n = seq_lens ? seq_lens[b] : ctx_len;
  g.n = g.n < 0 ? 0 : (g.n > ctx_len ? ctx_len : g.n);
  g.win_start = g.n - window > 0 ? g.n - window : 0;
  g.sink_end = n_sink < g.win_start ? n_sink : g.win_start;
  g.ncand = g.win_start - g.sink_end;
  return g;
}

// One query head.  T: row element type (uint16_t = bf16, float).
template <typename T, typename Ops>
void attend_head(const a2ats_dims& d, int b, int h, const T* q, const float* q_rot, const T* k_cache, const T* v_cache,
                 const int32_t* topk_idx, const int32_t* topk_count, int top_k, int window, int n_sink,
                 const float* cos_win, const float* sin_win, const int32_t* seq_lens, T* out) {
  const int Hq = d.n_q_heads, Hkv = d.n_kv_heads, G = Hq / Hkv, kv = h / G, bh = b * Hq + h;
  const Geometry g = geometry(d.ctx_len, seq_lens, b, window, n_sink);
  T* o = out + (size_t)bh * kD;
  if (g.n == 0) {
    for (int i = 0; i < kD; ++i) o[i] = T(0);
    return;
  }
  int cnt = topk_count[bh];
  cnt = std::max(0, std::min(std::min(cnt, top_k), g.ncand));
  const int n_far = g.sink_end + cnt, n_win = g.n - g.win_start, n_rows = n_far + n_win;
  const size_t seq = ((size_t)b * Hkv + kv) * (size_t)d.ctx_stride * kD;
  const T* kb = k_cache + seq;
  const T* vb = v_cache + seq;
  const int32_t* idx = topk_idx + (size_t)bh * top_k;
  const float* qr = q_rot + (size_t)bh * kD;
  float qf[kD];   // the raw query widened (window rows rotate it per row)
  for (int i = 0; i < kD; ++i) {
    if (sizeof(T) == 2) qf[i] = bf16_to_f32(((const uint16_t*)q)[(size_t)bh * kD + i]);
    else qf[i] = ((const float*)q)[(size_t)bh * kD + i];
  }
  const float scale = 0.08838834764831845f;   // 1/sqrt(128)
  auto row_of = [&](int t) {                  // t-th attended row: sinks, retrieved, window
    int j;
    if (t < g.sink_end) j = t;
    else if (t < n_far) j = idx[t - g.sink_end];
    else j = g.win_start + (t - n_far);
    return std::min(std::max(j, 0), g.n - 1);   // a bad caller index must not leave the cache
  };

  float m_run = -INFINITY, l_run = 0.f;
  alignas(32) float acc[kD];
  for (int i = 0; i < kD; ++i) acc[i] = 0.f;
  int rows[kBlock], next_rows[kBlock];
  int nb = std::min(kBlock, n_rows);
  for (int i = 0; i < nb; ++i) {
    rows[i] = row_of(i);
    prefetch_row(kb + (size_t)rows[i] * kD, kD * sizeof(T));
    prefetch_row(vb + (size_t)rows[i] * kD, kD * sizeof(T));
  }
  for (int t0 = 0; t0 < n_rows; t0 += kBlock) {
    const int nn = std::min(kBlock, n_rows - t0 - nb);   // the block after this one: request it now
    for (int i = 0; i < nn; ++i) {
      next_rows[i] = row_of(t0 + nb + i);
      prefetch_row(kb + (size_t)next_rows[i] * kD, kD * sizeof(T));
      prefetch_row(vb + (size_t)next_rows[i] * kD, kD * sizeof(T));
    }
    float logit[kBlock];
    float m_blk = -INFINITY;
    for (int i = 0; i < nb; ++i) {
      const int t = t0 + i, j = rows[i];
      const T* kr = kb + (size_t)j * kD;
      float dot;
      if (t < n_far) {
        dot = Ops::dot(qr, kr);
      } else {   // window row: (q R_delta) . k with the rotation at the relative position delta = n - 1 - j
        const int delta = std::min(std::max(g.n - 1 - j, 0), window - 1);
        const float* c = cos_win + (size_t)delta * (kD / 2);
        const float* s = sin_win + (size_t)delta * (kD / 2);
        alignas(32) float qd[kD];
        for (int u = 0; u < kD / 2; ++u) {
          qd[u] = qf[u] * c[u] - qf[u + kD / 2] * s[u];
          qd[u + kD / 2] = qf[u + kD / 2] * c[u] + qf[u] * s[u];
        }
        dot = Ops::dot(qd, kr);
      }
      logit[i] = dot * scale;
      m_blk = std::max(m_blk, logit[i]);
    }
    const float m_new = std::max(m_run, m_blk);
    const float alpha = expf(m_run - m_new);   // 0 for the first block
    if (alpha != 1.f) Ops::scale(acc, alpha);
    l_run *= alpha;
    for (int i = 0; i < nb; ++i) {
      const float p = expf(logit[i] - m_new);
      l_run += p;
      Ops::axpy(acc, p, vb + (size_t)rows[i] * kD);
    }
    m_run = m_new;
    nb = nn;
    for (int i = 0; i < nn; ++i) rows[i] = next_rows[i];
  }
  for (int i = 0; i < kD; ++i) {
    const float v = l_run > 0.f ? acc[i] / l_run : 0.f;
    if (sizeof(T) == 2) ((uint16_t*)o)[i] = f32_to_bf16(v);
    else ((float*)o)[i] = v;
  }
}

template <typename T>
void attend_all(const a2ats_dims& d, const void* q, const float* q_rot, const void* k_cache, const void* v_cache,
                const int32_t* topk_idx, const int32_t* topk_count, int top_k, int window, int n_sink,
                const float* cos_win, const float* sin_win, const int32_t* seq_lens, void* out, int n_threads) {
  const int heads = d.batch * d.n_q_heads;
  bool avx2 = false;
#if defined(__x86_64__)
  avx2 = __builtin_cpu_supports("avx2") && __builtin_cpu_supports("fma");
#endif
  if (n_threads < 1) n_threads = omp_get_max_threads();
#pragma omp parallel for schedule(dynamic, 1) num_threads(n_threads)
  for (int bh = 0; bh < heads; ++bh) {
    const int b = bh / d.n_q_heads, h = bh % d.n_q_heads;
#if defined(__x86_64__)
    if (avx2) {
      attend_head<T, Avx2Ops>(d, b, h, (const T*)q, q_rot, (const T*)k_cache, (const T*)v_cache, topk_idx, topk_count,
                              top_k, window, n_sink, cos_win, sin_win, seq_lens, (T*)out);
      continue;
    }
#endif
    attend_head<T, ScalarOps>(d, b, h, (const T*)q, q_rot, (const T*)k_cache, (const T*)v_cache, topk_idx, topk_count,
                              top_k, window, n_sink, cos_win, sin_win, seq_lens, (T*)out);
  }
}

}  // namespace

extern "C" int a2ats_sparse_attn_host(const a2ats_dims* d, const void* q, const float* q_rot, const void* k_cache,
                                      const void* v_cache, int kv_dtype, const int32_t* topk_idx,
                                      const int32_t* topk_count, int32_t top_k, int32_t window, int32_t n_sink,
                                      const float* cos_win, const float* sin_win, const int32_t* seq_lens, void* out,
                                      int32_t n_threads) {
  if (!d) return A2ATS_ERR_INVALID_ARG;
  if (d->batch < 0 || d->n_q_heads < 1 || d->n_kv_heads < 1 || d->n_q_heads % d->n_kv_heads != 0 || d->ctx_len < 0 ||
      d->ctx_stride < d->ctx_len)
    return A2ATS_ERR_INVALID_ARG;
  if (d->head_dim != kD) return A2ATS_ERR_UNSUPPORTED;
  if (top_k < 0 || window < 0 || n_sink < 0 || n_threads < 0) return A2ATS_ERR_INVALID_ARG;
  if (kv_dtype != A2ATS_F32 && kv_dtype != A2ATS_BF16) return A2ATS_ERR_INVALID_ARG;
  if (!q || !q_rot || !k_cache || !v_cache || !topk_count || !out) return A2ATS_ERR_INVALID_ARG;
  if (top_k > 0 && !topk_idx) return A2ATS_ERR_INVALID_ARG;
  if (window > 0 && (!cos_win || !sin_win)) return A2ATS_ERR_INVALID_ARG;
  if (kv_dtype == A2ATS_BF16)
    attend_all<uint16_t>(*d, q, q_rot, k_cache, v_cache, topk_idx, topk_count, top_k, window, n_sink, cos_win, sin_win,
                         seq_lens, out, n_threads);
  else
    attend_all<float>(*d, q, q_rot, k_cache, v_cache, topk_idx, topk_count, top_k, window, n_sink, cos_win, sin_win,
                      seq_lens, out, n_threads);
  return A2ATS_OK;
}
