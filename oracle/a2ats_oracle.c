/*
 * CPU oracle for the A2ATS decode-time retrieval path (arXiv 2502.12665).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what the
 * path computes, written from the paper's definitions in double precision.  It
 * shares no code, header, table or constant with the HIP library and must never
 * be linked into, imported by or called from the product path; only the tests,
 * the smoke check and the benchmark's CPU-baseline leg use it.
 *
 * Every routine takes the given inputs as float32 arrays (bf16 inputs are
 * widened exactly by the caller) and does all arithmetic in float64.  There is
 * no blocking, fusion or reordering beyond the definition; the only concession
 * to run time is an OpenMP "parallel for" over independent (batch, head)
 * problems.
 *
 * Layout conventions (row-major, last index fastest):
 *   q, out        [B, Hq, D]
 *   codebook      [Hkv, M, L, ds]     (M*ds == D; subspace m covers dims m*ds .. m*ds+ds-1)
 *   codes         [B, Hkv, S, M]      uint8 (code_bytes == 1) or uint16 (code_bytes == 2, for codebooks
 *                                     of more than 256 codewords: section 5.1 uses 4096 per head with
 *                                     M == 1), S = token-axis capacity >= N
 *   k, v          [B, Hkv, S, D]
 *   scores        [B, Hq, N]
 *   topk_idx      [B, Hq, K]          ascending token index, unused slots = -1
 * Query head h reads KV head h / G, G = Hq / Hkv.  Positions are 0-based; a
 * sequence of n tokens has its current (query) token at position i = n - 1,
 * and its key/value/code are already in the cache.
 *
 * Readings of the paper taken here (the paper is silent on them):
 *   - RoPE pairs dimension t with t + D/2 (the convention of the Llama / Mistral /
 *     Qwen families the paper evaluates), angle = position * inv_freq[t].
 *   - The window is {j : i - j < w}, i.e. the last w tokens including the current one
 *     (eq. "WRoPE", section 4.1); sinks are the first n_sink tokens (appendix A).
 *   - Top-K candidates are the tokens that are neither sinks nor in the window;
 *     selection is per query head; equal scores go to the lowest token index.
 *   - Approximate scores are not scaled; 1/sqrt(D) is applied in the attention only.
 *
 * Parity pins for every routine live in tests/test_oracle_pins.py; none is unpinned.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

static inline int code_at(const void *codes, int64_t i, int code_bytes) {
  return code_bytes == 2 ? (int)((const uint16_t *)codes)[i] : (int)((const uint8_t *)codes)[i];
}
static inline void code_put(void *codes, int64_t i, int code_bytes, int c) {
  if (code_bytes == 2) ((uint16_t *)codes)[i] = (uint16_t)c;
  else ((uint8_t *)codes)[i] = (uint8_t)c;
}

int a2ats_oracle_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* ---------------------------------------------------------------------------
 * O1. Rotary position embedding x -> x R_pos (section 2.1, eq. "rope").
 * R_pos rotates each pair (x[t], x[t + D/2]) by the angle pos * inv_freq[t].
 * The WRoPE query of section 4.1 is rope(q, b); WRoPE keys are rope(k, 0) = k.
 * ------------------------------------------------------------------------- */
static void rope_one(const float *x, int D, const double *inv_freq, double pos, double *out) {
  int half = D / 2;
  for (int t = 0; t < half; ++t) {
    double ang = pos * inv_freq[t];
    double c = cos(ang), s = sin(ang);
    double x1 = (double)x[t], x2 = (double)x[t + half];
    out[t] = x1 * c - x2 * s;
    out[t + half] = x2 * c + x1 * s;
  }
}

int a2ats_oracle_rope(const float *x, int64_t rows, int D, const double *inv_freq, double pos,
                      double *out) {
  for (int64_t r = 0; r < rows; ++r) rope_one(x + r * D, D, inv_freq, pos, out + r * D);
  return 0;
}

/* ---------------------------------------------------------------------------
 * O2a. Approximate score by definition (section 2.2 eq. "attention weights
 * approximation", section 4.2 last equation): rebuild the quantised key
 * k^_j = concat_m codebook[kv, m, codes[j, m], :] and take the D-term dot
 * product with the WRoPE query q~ (q_rot, float64, [B,Hq,D]).
 * ------------------------------------------------------------------------- */
int a2ats_oracle_scores_explicit(const double *q_rot, const float *codebook, const void *codes,
                                 int code_bytes, int B, int Hq, int Hkv, int M, int L, int ds, int64_t N,
                                 int64_t S, double *scores) {
  int D = M * ds, G = Hq / Hkv;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
  for (int b = 0; b < B; ++b)
    for (int h = 0; h < Hq; ++h) {
      int kv = h / G;
      const double *qr = q_rot + ((int64_t)b * Hq + h) * D;
      double *khat = (double *)malloc(sizeof(double) * D);
      for (int64_t j = 0; j < N; ++j) {
        const int64_t row = (((int64_t)b * Hkv + kv) * S + j) * M;
        for (int m = 0; m < M; ++m) {
          const float *c = codebook + (((int64_t)kv * M + m) * L + code_at(codes, row + m, code_bytes)) * ds;
          for (int t = 0; t < ds; ++t) khat[m * ds + t] = (double)c[t];
        }
        double u = 0.0;
        for (int d = 0; d < D; ++d) u += qr[d] * khat[d];
        scores[((int64_t)b * Hq + h) * N + j] = u;
      }
      free(khat);
    }
  return 0;
}

/* ---------------------------------------------------------------------------
 * O2b. The same score through per-subspace lookup tables:
 * lut[b,h,m,c] = sum_t q~[m*ds+t] * codebook[kv,m,c,t];  u^_j = sum_m lut[m, codes[j,m]].
 * Used to pin O2a (the two must agree to rounding) and as the statement of the
 * table the library builds.
 * ------------------------------------------------------------------------- */
int a2ats_oracle_lut(const double *q_rot, const float *codebook, int B, int Hq, int Hkv, int M,
                     int L, int ds, double *lut) {
  int D = M * ds, G = Hq / Hkv;
  for (int b = 0; b < B; ++b)
    for (int h = 0; h < Hq; ++h) {
      int kv = h / G;
      const double *qr = q_rot + ((int64_t)b * Hq + h) * D;
      for (int m = 0; m < M; ++m)
        for (int c = 0; c < L; ++c) {
          const float *cw = codebook + (((int64_t)kv * M + m) * L + c) * ds;
          double acc = 0.0;
          for (int t = 0; t < ds; ++t) acc += qr[m * ds + t] * (double)cw[t];
          lut[(((int64_t)b * Hq + h) * M + m) * L + c] = acc;
        }
    }
  return 0;
}

int a2ats_oracle_scores_lut(const double *lut, const void *codes, int code_bytes, int B, int Hq,
                            int Hkv, int M, int L, int64_t N, int64_t S, double *scores) {
  int G = Hq / Hkv;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
  for (int b = 0; b < B; ++b)
    for (int h = 0; h < Hq; ++h) {
      int kv = h / G;
      const double *t = lut + ((int64_t)b * Hq + h) * M * L;
      for (int64_t j = 0; j < N; ++j) {
        const int64_t row = (((int64_t)b * Hkv + kv) * S + j) * M;
        double u = 0.0;
        for (int m = 0; m < M; ++m) u += t[(int64_t)m * L + code_at(codes, row + m, code_bytes)];
        scores[((int64_t)b * Hq + h) * N + j] = u;
      }
    }
  return 0;
}

/* ---------------------------------------------------------------------------
 * O3. Top-K retrieval (section 4, "retrieves the top-K tokens with the highest
 * attention scores") by a full sort.  For a sequence of n tokens the candidates
 * are the positions [sink_end, n - w) with sink_end = min(n_sink, max(0, n - w));
 * they are ordered by (score descending, index ascending), the first
 * K' = min(K, #candidates) are taken and returned in ascending index order.
 * kth_score receives the K'-th largest score (NaN when K' == 0).
 * seq_lens (nullable, [B]) gives n per sequence; otherwise n = N.
 * ------------------------------------------------------------------------- */
typedef struct {
  double s;
  int32_t j;
} scored_t;

static int cmp_score_desc_idx_asc(const void *a, const void *b) {
  const scored_t *x = (const scored_t *)a, *y = (const scored_t *)b;
  if (x->s > y->s) return -1;
  if (x->s < y->s) return 1;
  return (x->j > y->j) - (x->j < y->j);
}

static int cmp_i32(const void *a, const void *b) {
  int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
  return (x > y) - (x < y);
}

int a2ats_oracle_topk(const double *scores, int B, int Hq, int64_t N, int K, int w, int n_sink,
                      const int32_t *seq_lens, int32_t *topk_idx, int32_t *topk_count,
                      double *kth_score) {
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
  for (int b = 0; b < B; ++b)
    for (int h = 0; h < Hq; ++h) {
      int64_t n = seq_lens ? seq_lens[b] : N;
      int64_t win_start = n - w > 0 ? n - w : 0;
      int64_t sink_end = n_sink < win_start ? n_sink : win_start;
      int64_t ncand = win_start - sink_end;
      int64_t kk = K < ncand ? K : ncand;
      int32_t *out = topk_idx + ((int64_t)b * Hq + h) * K;
      for (int t = 0; t < K; ++t) out[t] = -1;
      topk_count[(int64_t)b * Hq + h] = (int32_t)kk;
      kth_score[(int64_t)b * Hq + h] = NAN;
      if (kk <= 0) continue;
      scored_t *arr = (scored_t *)malloc(sizeof(scored_t) * (size_t)ncand);
      const double *s = scores + ((int64_t)b * Hq + h) * N;
      for (int64_t t = 0; t < ncand; ++t) {
        arr[t].s = s[sink_end + t];
        arr[t].j = (int32_t)(sink_end + t);
      }
      qsort(arr, (size_t)ncand, sizeof(scored_t), cmp_score_desc_idx_asc);
      for (int64_t t = 0; t < kk; ++t) out[t] = arr[t].j;
      kth_score[(int64_t)b * Hq + h] = arr[kk - 1].s;
      qsort(out, (size_t)kk, sizeof(int32_t), cmp_i32);
      free(arr);
    }
  return 0;
}

/* ---------------------------------------------------------------------------
 * O4a. Selective attention under WRoPE (section 2.1 eq. "output state" restricted
 * to the attended set, section 4.1 eq. "WRoPE").  For query position i = n - 1:
 *   logit_j = q R_{i-j} k_j^T / sqrt(D)   if i - j <  w   (window: standard RoPE)
 *   logit_j = q R_b     k_j^T / sqrt(D)   if i - j >= w   (retrieved tokens and sinks)
 * over S = sinks U top-K U window; out = sum_j softmax(logit)_j v_j.
 * Keys are the exact pre-RoPE keys (WRoPE leaves keys unrotated).
 * ------------------------------------------------------------------------- */
static void attend_set(const float *q, const float *kbase, const float *vbase, int D,
                       const int64_t *set, int64_t nset, int64_t i, int w, double b_off,
                       const double *inv_freq, double *out) {
  double *logit = (double *)malloc(sizeof(double) * (size_t)(nset > 0 ? nset : 1));
  double *qr = (double *)malloc(sizeof(double) * D);
  double mx = -INFINITY;
  for (int64_t t = 0; t < nset; ++t) {
    int64_t j = set[t];
    double pos = (i - j < w) ? (double)(i - j) : b_off;
    rope_one(q, D, inv_freq, pos, qr);
    const float *kj = kbase + j * D;
    double u = 0.0;
    for (int d = 0; d < D; ++d) u += qr[d] * (double)kj[d];
    logit[t] = u / sqrt((double)D);
    if (logit[t] > mx) mx = logit[t];
  }
  double den = 0.0;
  for (int64_t t = 0; t < nset; ++t) {
    logit[t] = exp(logit[t] - mx);
    den += logit[t];
  }
  for (int d = 0; d < D; ++d) out[d] = 0.0;
  for (int64_t t = 0; t < nset; ++t) {
    const float *vj = vbase + set[t] * D;
    double p = logit[t] / den;
    for (int d = 0; d < D; ++d) out[d] += p * (double)vj[d];
  }
  free(logit);
  free(qr);
}

int a2ats_oracle_sparse_attn(const float *q, const float *k, const float *v,
                             const int32_t *topk_idx, const int32_t *topk_count, int B, int Hq,
                             int Hkv, int D, int64_t N, int64_t S, int K, int w, int n_sink,
                             const double *inv_freq, double b_off, const int32_t *seq_lens,
                             double *out) {
  int G = Hq / Hkv;
  int bad = 0;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
  for (int b = 0; b < B; ++b)
    for (int h = 0; h < Hq; ++h) {
      int kv = h / G;
      int64_t n = seq_lens ? seq_lens[b] : N;
      double *o = out + ((int64_t)b * Hq + h) * D;
      if (n <= 0) {
        for (int d = 0; d < D; ++d) o[d] = 0.0;
        continue;
      }
      int64_t win_start = n - w > 0 ? n - w : 0;
      int64_t sink_end = n_sink < win_start ? n_sink : win_start;
      int cnt = topk_count[(int64_t)b * Hq + h];
      int64_t nset = sink_end + cnt + (n - win_start);
      int64_t *set = (int64_t *)malloc(sizeof(int64_t) * (size_t)nset);
      int64_t p = 0;
      for (int64_t j = 0; j < sink_end; ++j) set[p++] = j;
      for (int t = 0; t < cnt; ++t) {
        int64_t j = topk_idx[((int64_t)b * Hq + h) * K + t];
        if (j < sink_end || j >= win_start) {
#pragma omp atomic write
          bad = 1;
          j = sink_end;
        }
        set[p++] = j;
      }
      for (int64_t j = win_start; j < n; ++j) set[p++] = j;
      attend_set(q + ((int64_t)b * Hq + h) * D, k + ((int64_t)b * Hkv + kv) * S * D,
                 v + ((int64_t)b * Hkv + kv) * S * D, D, set, nset, n - 1, w, b_off, inv_freq, o);
      free(set);
    }
  return bad ? -1 : 0;
}

/* O4b. Dense attention over every cached token j <= i under eq. "WRoPE".  With
 * w >= n it is standard RoPE attention; O4a with K >= n - w must reproduce it. */
int a2ats_oracle_dense_wrope_attn(const float *q, const float *k, const float *v, int B, int Hq,
                                  int Hkv, int D, int64_t N, int64_t S, int w,
                                  const double *inv_freq, double b_off, const int32_t *seq_lens,
                                  double *out) {
  int G = Hq / Hkv;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
  for (int b = 0; b < B; ++b)
    for (int h = 0; h < Hq; ++h) {
      int kv = h / G;
      int64_t n = seq_lens ? seq_lens[b] : N;
      double *o = out + ((int64_t)b * Hq + h) * D;
      if (n <= 0) {
        for (int d = 0; d < D; ++d) o[d] = 0.0;
        continue;
      }
      int64_t *set = (int64_t *)malloc(sizeof(int64_t) * (size_t)n);
      for (int64_t j = 0; j < n; ++j) set[j] = j;
      attend_set(q + ((int64_t)b * Hq + h) * D, k + ((int64_t)b * Hkv + kv) * S * D,
                 v + ((int64_t)b * Hkv + kv) * S * D, D, set, n, n - 1, w, b_off, inv_freq, o);
      free(set);
    }
  return 0;
}

/* ---------------------------------------------------------------------------
 * O5a. Key encoding (section 2.2 quantisation function f; section 4.2 query-aware
 * f'):  code[j,m] = argmin_c (k_m - C[m,c]) H_m (k_m - C[m,c])^T, scanning
 * c = 0..L-1 with a strict "<" so the lowest index wins exact ties.
 *   mode 0: H_m = I (plain nearest centroid), weights ignored
 *   mode 1: H_m = diag(weights[kv, m*ds .. m*ds+ds-1]),  weights [Hkv, D]
 *   mode 2: H_m = weights[kv, m, :, :] (ds x ds, symmetric PD), weights [Hkv, M, ds, ds]
 * best/second (nullable, [B,Hkv,n,M]) receive the smallest and second smallest
 * distortion so a caller can recognise near-ties.
 * ------------------------------------------------------------------------- */
static double quad_form(const double *d, const float *Hm, int ds, int mode) {
  double acc = 0.0;
  if (mode == 0) {
    for (int t = 0; t < ds; ++t) acc += d[t] * d[t];
  } else if (mode == 1) {
    for (int t = 0; t < ds; ++t) acc += d[t] * (double)Hm[t] * d[t];
  } else {
    for (int r = 0; r < ds; ++r)
      for (int c = 0; c < ds; ++c) acc += d[r] * (double)Hm[r * ds + c] * d[c];
  }
  return acc;
}

int a2ats_oracle_encode(const float *keys, const float *codebook, const float *weights, int mode,
                        int B, int Hkv, int64_t n, int M, int L, int ds, void *codes, int code_bytes,
                        double *best, double *second) {
  int D = M * ds;
  if (ds > 128) return -2;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
  for (int b = 0; b < B; ++b)
    for (int kv = 0; kv < Hkv; ++kv) {
      double d[128];
      for (int64_t j = 0; j < n; ++j) {
        const float *key = keys + (((int64_t)b * Hkv + kv) * n + j) * D;
        for (int m = 0; m < M; ++m) {
          const float *Hm = NULL;
          if (mode == 1) Hm = weights + (int64_t)kv * D + m * ds;
          if (mode == 2) Hm = weights + ((int64_t)kv * M + m) * ds * ds;
          double b1 = INFINITY, b2 = INFINITY;
          int arg = 0;
          for (int c = 0; c < L; ++c) {
            const float *cw = codebook + (((int64_t)kv * M + m) * L + c) * ds;
            for (int t = 0; t < ds; ++t) d[t] = (double)key[m * ds + t] - (double)cw[t];
            double dist = quad_form(d, Hm, ds, mode);
            if (dist < b1) {
              b2 = b1;
              b1 = dist;
              arg = c;
            } else if (dist < b2) {
              b2 = dist;
            }
          }
          int64_t o = (((int64_t)b * Hkv + kv) * n + j) * M + m;
          code_put(codes, o, code_bytes, arg);
          if (best) best[o] = b1;
          if (second) second[o] = b2;
        }
      }
    }
  return 0;
}

/* O5b. The same assignment through the Cholesky reformulation of section 4.2
 * (eq. "definition z" and the equations after it): H_m = L_m L_m^T, z = k_m L_m,
 * c^z = c L_m, f'(k; C) = f(z; C^z) with the plain Euclidean distance.
 * weights is the block form [Hkv, M, ds, ds].  Returns -1 if a block is not
 * positive definite. */
int a2ats_oracle_encode_cholesky(const float *keys, const float *codebook, const float *weights,
                                 int B, int Hkv, int64_t n, int M, int L, int ds, void *codes,
                                 int code_bytes, double *best, double *second) {
  int D = M * ds;
  int bad = 0;
  if (ds > 128) return -2;
  for (int kv = 0; kv < Hkv; ++kv)
    for (int m = 0; m < M; ++m) {
      const float *Hm = weights + ((int64_t)kv * M + m) * ds * ds;
      double *Lc = (double *)calloc((size_t)ds * ds, sizeof(double));
      for (int r = 0; r < ds; ++r)
        for (int c = 0; c <= r; ++c) {
          double s = (double)Hm[r * ds + c];
          for (int t = 0; t < c; ++t) s -= Lc[r * ds + t] * Lc[c * ds + t];
          if (r == c) {
            if (s <= 0.0) bad = 1;
            Lc[r * ds + c] = sqrt(s > 0.0 ? s : 1.0);
          } else {
            Lc[r * ds + c] = s / Lc[c * ds + c];
          }
        }
      double *cz = (double *)malloc(sizeof(double) * L * ds);
      for (int c = 0; c < L; ++c) {
        const float *cw = codebook + (((int64_t)kv * M + m) * L + c) * ds;
        for (int t = 0; t < ds; ++t) {
          double s = 0.0;
          for (int r = 0; r < ds; ++r) s += (double)cw[r] * Lc[r * ds + t];
          cz[c * ds + t] = s;
        }
      }
#pragma omp parallel for schedule(static)
      for (int b = 0; b < B; ++b)
        for (int64_t j = 0; j < n; ++j) {
          const float *key = keys + (((int64_t)b * Hkv + kv) * n + j) * D + m * ds;
          double z[128];
          for (int t = 0; t < ds; ++t) {
            double s = 0.0;
            for (int r = 0; r < ds; ++r) s += (double)key[r] * Lc[r * ds + t];
            z[t] = s;
          }
          double b1 = INFINITY, b2 = INFINITY;
          int arg = 0;
          for (int c = 0; c < L; ++c) {
            double dist = 0.0;
            for (int t = 0; t < ds; ++t) {
              double e = z[t] - cz[c * ds + t];
              dist += e * e;
            }
            if (dist < b1) {
              b2 = b1;
              b1 = dist;
              arg = c;
            } else if (dist < b2) {
              b2 = dist;
            }
          }
          int64_t o = (((int64_t)b * Hkv + kv) * n + j) * M + m;
          code_put(codes, o, code_bytes, arg);
          if (best) best[o] = b1;
          if (second) second[o] = b2;
        }
      free(cz);
      free(Lc);
    }
  return bad ? -1 : 0;
}
