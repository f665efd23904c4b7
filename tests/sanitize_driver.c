/* Small-case driver for the CPU oracle built with -fsanitize=address,undefined (host code only).
 * It calls every routine of oracle/a2ats_oracle.c on small seeded inputs with ragged lengths,
 * sinks, empty sequences and 16-bit codes, in exactly sized heap buffers, so that an out-of-bounds
 * access, an uninitialised-size slip or undefined arithmetic inside the oracle aborts the run.  It also
 * re-checks three of the oracle's pins on the way (table route == explicit route, K >= n - w gives the
 * dense result, the two encoder forms agree), and prints "sanitize ok" at the end. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int a2ats_oracle_rope(const float *x, int64_t rows, int D, const double *inv_freq, double pos, double *out);
int a2ats_oracle_scores_explicit(const double *q_rot, const float *codebook, const void *codes, int code_bytes,
                                 int B, int Hq, int Hkv, int M, int L, int ds, int64_t N, int64_t S, double *scores);
int a2ats_oracle_lut(const double *q_rot, const float *codebook, int B, int Hq, int Hkv, int M, int L, int ds,
                     double *lut);
int a2ats_oracle_scores_lut(const double *lut, const void *codes, int code_bytes, int B, int Hq, int Hkv, int M,
                            int L, int64_t N, int64_t S, double *scores);
int a2ats_oracle_topk(const double *scores, int B, int Hq, int64_t N, int K, int w, int n_sink,
                      const int32_t *seq_lens, int32_t *topk_idx, int32_t *topk_count, double *kth_score);
int a2ats_oracle_sparse_attn(const float *q, const float *k, const float *v, const int32_t *topk_idx,
                             const int32_t *topk_count, int B, int Hq, int Hkv, int D, int64_t N, int64_t S, int K,
                             int w, int n_sink, const double *inv_freq, double b_off, const int32_t *seq_lens,
                             double *out);
int a2ats_oracle_dense_wrope_attn(const float *q, const float *k, const float *v, int B, int Hq, int Hkv, int D,
                                  int64_t N, int64_t S, int w, const double *inv_freq, double b_off,
                                  const int32_t *seq_lens, double *out);
int a2ats_oracle_encode(const float *keys, const float *codebook, const float *weights, int mode, int B, int Hkv,
                        int64_t n, int M, int L, int ds, void *codes, int code_bytes, double *best, double *second);
int a2ats_oracle_encode_cholesky(const float *keys, const float *codebook, const float *weights, int B, int Hkv,
                                 int64_t n, int M, int L, int ds, void *codes, int code_bytes, double *best,
                                 double *second);

static uint64_t g_state = 88172645463325252ull;
static double unif(void) {   /* xorshift64: uniform in (0, 1) */
  g_state ^= g_state << 13; g_state ^= g_state >> 7; g_state ^= g_state << 17;
  return ((double)(g_state >> 11) + 0.5) / 9007199254740992.0;
}
static float gauss(void) { return (float)(sqrt(-2.0 * log(unif())) * cos(6.283185307179586 * unif())); }
static void *xmalloc(size_t n) { void *p = malloc(n ? n : 1); if (!p) { fprintf(stderr, "out of memory\n"); exit(2); } return p; }
#define CHECK(c) do { if (!(c)) { fprintf(stderr, "check failed at line %d: %s\n", __LINE__, #c); exit(1); } } while (0)

static void decode_case(int B, int Hq, int Hkv, int M, int L, int ds, int N, int S, int K, int w, int n_sink,
                        const int32_t *lens, int code_bytes) {
  const int D = M * ds;
  float *q = xmalloc(sizeof(float) * B * Hq * D), *cb = xmalloc(sizeof(float) * Hkv * M * L * ds);
  float *k = xmalloc(sizeof(float) * B * Hkv * S * D), *v = xmalloc(sizeof(float) * B * Hkv * S * D);
  double *inv = xmalloc(sizeof(double) * (D / 2)), *qrot = xmalloc(sizeof(double) * B * Hq * D);
  void *codes = xmalloc((size_t)code_bytes * B * Hkv * S * M);
  for (int i = 0; i < B * Hq * D; ++i) q[i] = gauss();
  for (int i = 0; i < Hkv * M * L * ds; ++i) cb[i] = gauss();
  for (int64_t i = 0; i < (int64_t)B * Hkv * S * D; ++i) { k[i] = gauss(); v[i] = gauss(); }
  for (int t = 0; t < D / 2; ++t) inv[t] = pow(10000.0, -2.0 * t / D);
  for (int64_t i = 0; i < (int64_t)B * Hkv * S * M; ++i) {
    const unsigned c = (unsigned)(unif() * L) % (unsigned)L;
    if (code_bytes == 1) ((uint8_t *)codes)[i] = (uint8_t)c; else ((uint16_t *)codes)[i] = (uint16_t)c;
  }
  CHECK(a2ats_oracle_rope(q, (int64_t)B * Hq, D, inv, 2048.0, qrot) == 0);
  double *s1 = xmalloc(sizeof(double) * B * Hq * N), *s2 = xmalloc(sizeof(double) * B * Hq * N);
  double *lut = xmalloc(sizeof(double) * B * Hq * M * L);
  CHECK(a2ats_oracle_scores_explicit(qrot, cb, codes, code_bytes, B, Hq, Hkv, M, L, ds, N, S, s1) == 0);
  CHECK(a2ats_oracle_lut(qrot, cb, B, Hq, Hkv, M, L, ds, lut) == 0);
  CHECK(a2ats_oracle_scores_lut(lut, codes, code_bytes, B, Hq, Hkv, M, L, N, S, s2) == 0);
  for (int i = 0; i < B * Hq * N; ++i) CHECK(fabs(s1[i] - s2[i]) <= 1e-12 * (1.0 + fabs(s1[i])));
  int32_t *idx = xmalloc(sizeof(int32_t) * B * Hq * (K ? K : 1)), *cnt = xmalloc(sizeof(int32_t) * B * Hq);
  double *kth = xmalloc(sizeof(double) * B * Hq), *out = xmalloc(sizeof(double) * B * Hq * D);
  double *dense = xmalloc(sizeof(double) * B * Hq * D);
  CHECK(a2ats_oracle_topk(s1, B, Hq, N, K, w, n_sink, lens, idx, cnt, kth) == 0);
  for (int bh = 0; bh < B * Hq; ++bh) {
    const int n = lens ? lens[bh / Hq] : N;
    const int ws = n - w > 0 ? n - w : 0, se = n_sink < ws ? n_sink : ws;
    CHECK(cnt[bh] == (K < ws - se ? K : ws - se));
    for (int t = 0; t < cnt[bh]; ++t) CHECK(idx[bh * K + t] >= se && idx[bh * K + t] < ws);
  }
  CHECK(a2ats_oracle_sparse_attn(q, k, v, idx, cnt, B, Hq, Hkv, D, N, S, K, w, n_sink, inv, 2048.0, lens, out) == 0);
  CHECK(a2ats_oracle_dense_wrope_attn(q, k, v, B, Hq, Hkv, D, N, S, w, inv, 2048.0, lens, dense) == 0);
  if (K >= N)   /* every candidate retrieved: selective == dense (section 4.1) */
    for (int i = 0; i < B * Hq * D; ++i) CHECK(fabs(out[i] - dense[i]) <= 1e-10);
  free(q); free(cb); free(k); free(v); free(inv); free(qrot); free(codes); free(s1); free(s2); free(lut);
  free(idx); free(cnt); free(kth); free(out); free(dense);
}

static void encode_case(int B, int Hkv, int n, int M, int L, int ds, int code_bytes) {
  const int D = M * ds;
  float *keys = xmalloc(sizeof(float) * B * Hkv * n * D), *cb = xmalloc(sizeof(float) * Hkv * M * L * ds);
  float *hd = xmalloc(sizeof(float) * Hkv * D), *hb = xmalloc(sizeof(float) * Hkv * M * ds * ds);
  for (int i = 0; i < B * Hkv * n * D; ++i) keys[i] = gauss();
  for (int i = 0; i < Hkv * M * L * ds; ++i) cb[i] = gauss();
  for (int i = 0; i < Hkv * D; ++i) hd[i] = (float)(0.1 + unif());
  for (int kv = 0; kv < Hkv; ++kv)
    for (int m = 0; m < M; ++m) {   /* A A^T / ds + 0.05 I: symmetric positive definite */
      float a[16 * 16];
      for (int i = 0; i < ds * ds; ++i) a[i] = gauss();
      for (int i = 0; i < ds; ++i)
        for (int j = 0; j < ds; ++j) {
          double acc = i == j ? 0.05 : 0.0;
          for (int t = 0; t < ds; ++t) acc += (double)a[i * ds + t] * a[j * ds + t] / ds;
          hb[((kv * M + m) * ds + i) * ds + j] = (float)acc;
        }
    }
  const size_t nc = (size_t)B * Hkv * n * M;
  void *c0 = xmalloc(nc * code_bytes), *c1 = xmalloc(nc * code_bytes), *c2 = xmalloc(nc * code_bytes);
  double *b1 = xmalloc(sizeof(double) * nc), *b2 = xmalloc(sizeof(double) * nc);
  CHECK(a2ats_oracle_encode(keys, cb, NULL, 0, B, Hkv, n, M, L, ds, c0, code_bytes, NULL, NULL) == 0);
  CHECK(a2ats_oracle_encode(keys, cb, hd, 1, B, Hkv, n, M, L, ds, c1, code_bytes, b1, b2) == 0);
  CHECK(a2ats_oracle_encode(keys, cb, hb, 2, B, Hkv, n, M, L, ds, c1, code_bytes, b1, b2) == 0);
  CHECK(a2ats_oracle_encode_cholesky(keys, cb, hb, B, Hkv, n, M, L, ds, c2, code_bytes, NULL, NULL) == 0);
  for (size_t i = 0; i < nc; ++i) {   /* quadratic form == Cholesky form outside near-ties (section 4.2) */
    const unsigned x = code_bytes == 1 ? ((uint8_t *)c1)[i] : ((uint16_t *)c1)[i];
    const unsigned y = code_bytes == 1 ? ((uint8_t *)c2)[i] : ((uint16_t *)c2)[i];
    CHECK(x == y || b2[i] - b1[i] <= 1e-9 * (1.0 + b2[i]));
    CHECK(x < (unsigned)L);
  }
  free(keys); free(cb); free(hd); free(hb); free(c0); free(c1); free(c2); free(b1); free(b2);
}

int main(void) {
  const int32_t lens[3] = {57, 0, 9};
  decode_case(3, 4, 2, 4, 256, 4, 57, 61, 7, 8, 2, lens, 1);     /* ragged, an empty sequence, one inside the window */
  decode_case(2, 6, 2, 2, 256, 8, 40, 40, 64, 5, 0, NULL, 1);    /* K >= n: dense */
  decode_case(1, 2, 1, 1, 4096, 16, 33, 33, 0, 4, 1, NULL, 2);   /* one codebook of 4096, 16-bit codes, K = 0 */
  decode_case(1, 1, 1, 4, 256, 4, 1, 1, 3, 4, 0, NULL, 1);       /* a single token */
  encode_case(2, 2, 37, 4, 256, 4, 1);
  encode_case(1, 1, 5, 1, 4096, 16, 2);
  printf("sanitize ok\n");
  return 0;
}
