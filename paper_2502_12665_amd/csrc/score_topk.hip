// Step 3 of a decode step: approximate scores by gather-summing fixed-point table entries
// through the uint8 codes (section 4.2 last equation), and exact per-head top-K (section 4).
//
// Two routes, chosen on the host from the shape:
//
//  exact route (short contexts, very large K; also the in-kernel fallback of the fast route):
//  one workgroup per query head runs an MSB-first radix select over the 32-bit score keys by
//  re-streaming its sequence (<= 3 histogram passes), then one ordered pass that emits the
//  winners in ascending position, equal scores going to the lower position.
//
//  fast route (long contexts): the code matrix is streamed from HBM once, against a 16-bit
//  coarse copy of the tables, and only rows near the K-th score are ever scored exactly.
//    1. sample_threshold_kernel scores a sample of each sequence (about 1/16 of it, taken in
//       128-byte runs spread evenly over the candidates) with the coarse tables and derives, per
//       head, a coarse threshold below the K-th score with a 5-sigma margin (distribution-free
//       for independent rows: it only uses ranks of the sample).
//    2. stream_select_kernel streams all code rows: one 8-byte LDS read per code byte serves the
//       four heads of a group (two heads per 32-bit word, 16 bits each, so one integer add
//       accumulates two heads).  A row whose coarse score reaches the threshold of any of the
//       heads is written once -- its position and the two words of coarse scores, 12 bytes -- to
//       the segment of its tile (a run of 256..2048 consecutive rows scored by one wave) in HBM.
//    3. final_select_kernel (one workgroup per head) gathers its head's survivors (about 1.7 K)
//       in position order, finds the K-th largest COARSE score c_K among them exactly, and uses
//         exact score = base + (coarse << s) + rem,  0 <= rem < M 2^s
//       twice: a row with coarse >= c_K + M beats every row with coarse <= c_K, of which all but
//       at most K - 1 are, so it is a winner; a row with coarse <= c_K - M loses to the at least
//       K rows with coarse >= c_K.  Only the rows in between (a few dozen) are scored exactly,
//       from their code bytes and the head's 32-bit table, and ranked (score, then position).
//       Every row with coarse > c_K - M must be on the list, i.e. threshold <= c_K - M + 1; if
//       that fails, or a list is too short / too long / overflowed, or the band in between is
//       too large (the sample misled -- about 1e-6 per head for independent rows, more when
//       similar rows come in runs -- or the input is degenerate, e.g. all rows equal), the
//       workgroup runs the exact route for its head, so the result is always exact with respect
//       to the 32-bit scores.
#include <hip/hip_ext.h>
#include <math.h>

#include <algorithm>
#include <cmath>
#include "common.hpp"
#include "internal.hpp"
#include "coarse_score.hpp"

namespace a2ats {

constexpr int kExactThreads = 1024;
constexpr int kStreamThreads = 512;
constexpr int kStreamWaves = kStreamThreads / 64;
constexpr int kSampleThreads = 512;
constexpr int kSegMeta = 8;          // words of a segment header: rows, 4 per-head counts, padding
constexpr int kSampleRows = 1024;    // rows scored by one sampling workgroup
constexpr int kTileUnit = 256;       // rows a wave scores per step (4 per lane)
constexpr int kMaxTiles = 512;       // tiles (= survivor segments) per problem the final kernel handles
constexpr int kEntryWords = 3;       // a survivor entry: position, coarse scores of heads 0|1, of heads 2|3
constexpr int kBandMax = 1024;       // rows within M coarse units of the K-th coarse score that are ranked exactly

TopkPlan make_topk_plan(const a2ats_dims& d, int top_k, int window, int n_sink) {
  TopkPlan p{};
  const int G = d.n_q_heads / d.n_kv_heads;
  p.NG = (G + kHeadsPerGroup - 1) / kHeadsPerGroup;
  long ncand = (long)d.ctx_len - window - n_sink;
  if (ncand < 0) ncand = 0;
  p.cap = 8192;
  p.fast = !single_codebook(d) && ncand >= 16384 && top_k >= 1 && top_k <= 2048 && 4L * top_k <= ncand;
  if (p.fast) {
    // Sample a sixteenth of the candidates, in units of kSampleRows, shared by at most 8
    // workgroups: up to 8 * kSampleRows each workgroup scores kSampleRows rows, beyond that (very
    // long contexts, where a small sample would put the 5-sigma threshold far too low and the
    // survivor lists would outgrow the final kernel's LDS) each takes an eighth of the sample.
    long s_tot = ncand / 16 / kSampleRows * kSampleRows;
    if (s_tot < kSampleRows) s_tot = kSampleRows;
    if (s_tot > 64 * kSampleRows) s_tot = 64 * kSampleRows;
    p.P0 = (int)std::min<long>(8, s_tot / kSampleRows);
    p.sample_rows = (int)(s_tot / p.P0);   // at most 8192: the histogram counts are 16 bits wide
    const long problems = (long)d.batch * d.n_kv_heads * p.NG;
    // Tiles: runs of tile_rows consecutive candidates, each scored by one wave and owning one
    // survivor segment; the segments of a problem taken in tile order are sorted by position.
    long tile_rows = (ncand + (long)kMaxTiles * kTileUnit - 1) / ((long)kMaxTiles * kTileUnit) * kTileUnit;
    const long n_tiles = (ncand + tile_rows - 1) / tile_rows;   // 64 .. 512
    // Workgroups: two per CU over the whole launch, each with at least one tile per wave.
    long chunks = (512 + problems - 1) / problems;
    const long max_chunks = (n_tiles + kStreamWaves - 1) / kStreamWaves;
    if (chunks > max_chunks) chunks = max_chunks;
    if (chunks < 1) chunks = 1;
    const long tpc = (n_tiles + chunks - 1) / chunks;
    chunks = (n_tiles + tpc - 1) / tpc;   // none empty
    // Survivor segments.  The sampling rule (rank r with r - 5 sqrt(r) >= K S / N, plus one per
    // part) lets about r N / S rows per head through -- for small K much more than K -- and a row
    // survives if any of the (up to) four heads wants it.  row_cap is twice that share of a tile's
    // rows plus 16 standard deviations of a Poisson count: survivors that come in runs
    // (neighbouring tokens with similar scores) scatter far more between tiles than independent
    // ones.  Unused capacity costs only scratch.
    const double r0 = (double)top_k * (double)s_tot / (double)ncand;
    const double xr = 0.5 * (kSigma + std::sqrt(kSigma * kSigma + 4.0 * r0));
    const double survivors = (xr * xr + 2.0 * p.P0) / (double)s_tot * (double)ncand * 1.25;
    const double keep = std::min(1.0, 4.0 * survivors / (double)ncand);
    const double mu = (double)tile_rows * keep;
    long cap_rows = (long)(mu * 2.0 + 16.0 * std::sqrt(mu)) + 64;
    cap_rows = (cap_rows + 31) / 32 * 32;
    if (cap_rows > tile_rows) cap_rows = tile_rows;
    p.chunks = (int)chunks;
    p.tile_rows = (int)tile_rows;
    p.n_tiles = (int)n_tiles;
    p.tiles_per_chunk = (int)tpc;
    p.row_cap = (int)cap_rows;                // a multiple of 32
    const size_t heads = (size_t)d.batch * d.n_q_heads;
    const size_t segs = (size_t)problems * p.n_tiles;
    p.off_thr = 0;
    p.off_route = (p.off_thr + heads * p.P0 * sizeof(int32_t) + 255) / 256 * 256;
    p.off_count = (p.off_route + heads * sizeof(uint32_t) + 255) / 256 * 256;
    p.off_cand = (p.off_count + segs * kSegMeta * sizeof(uint32_t) + 255) / 256 * 256;
    p.bytes = (p.off_cand + segs * (size_t)p.row_cap * kEntryWords * sizeof(uint32_t) + 255) / 256 * 256;
  }
  return p;
}

// ------------------------------------------------------------------------------------------
// Scoring primitives
// ------------------------------------------------------------------------------------------

// Exact score of one token for one head.  The head's table sits in LDS with one 256-byte row per
// centroid id c; the 4-byte entry of subspace m is at byte m << 2 of the row (M = 32), or, for
// M = 16, twice: at m << 2 and at 64 + (m << 2).  LDS serves a 4-byte read 32 lanes at a time.
// Lane L visits the subspaces of its row in the order m = t ^ (L & 15) within a 16-byte half row,
// and lanes 16..31 of each half-wave use the second copy (M = 16) or take the two half rows in the
// other order (M = 32): the 32 lanes served together then touch 32 different banks whatever the
// code bytes are (a [m][c] table would spread them at random: ~3.5 lanes on the busiest bank).
// The visiting order does not change the result because the scores are integer sums.
constexpr int kExactLdsBytes = kCentroids * 256;

template <int M, int NT>
__device__ __forceinline__ void load_exact_table(const int32_t* __restrict__ head_table, unsigned char* tbl) {
  const int4* src = (const int4*)head_table;   // [256 c][M] int32
#pragma unroll 4
  for (int e = threadIdx.x; e < kCentroids * M / 4; e += NT) {
    const int c = e / (M / 4), mq = e % (M / 4);
    const int4 v = src[e];
    *(int4*)(tbl + (c << 8) + (mq << 4)) = v;
    if (M == 16) *(int4*)(tbl + (c << 8) + 64 + (mq << 4)) = v;
  }
}

template <int M>
struct ExactSwizzle {
  uint32_t mc[M / 4];   // byte t&3 of mc[t>>2]: low address byte for step t of this lane
  uint32_t sel[4];      // v_perm selectors: address byte 1 <- code byte (k ^ b), byte 0 <- mc byte k
  bool swap1, swap2;    // dword index inside a half row is XORed with (rho >> 2)
  bool swaph;           // M = 32: this lane takes the two half rows in the other order
  __device__ __forceinline__ void init(int lane) {
    const uint32_t rho = lane & 15, b = rho & 3, hi = (lane >> 4) & 1;
#pragma unroll
    for (int d = 0; d < M / 4; ++d) {
      uint32_t v = 0;
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const uint32_t t = 4 * d + k;
        const uint32_t m_low = (t ^ rho) & 15u, half = t >> 4;
        const uint32_t byte = M == 16 ? ((hi << 6) | (m_low << 2)) : ((((half ^ hi) << 4) | m_low) << 2);
        v |= byte << (8 * k);
      }
      mc[d] = v;
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) sel[k] = 0x0c0c0000u | ((4u + ((uint32_t)k ^ b)) << 8) | (uint32_t)k;
    swap1 = (rho >> 2) & 1;
    swap2 = (rho >> 3) & 1;
    swaph = M == 32 && hi;
  }
};

template <int M>
__device__ __forceinline__ int32_t score_exact(const uint4 (&w)[M / 16], const unsigned char* tbl,
                                               const ExactSwizzle<M>& sw) {
  int32_t s = 0;
#pragma unroll
  for (int qd = 0; qd < M / 16; ++qd) {
    uint4 h = w[qd];
    if (M == 32) {
      const uint4 o = w[(M / 16 - 1) - qd];
      h = make_uint4(sw.swaph ? o.x : h.x, sw.swaph ? o.y : h.y, sw.swaph ? o.z : h.z, sw.swaph ? o.w : h.w);
    }
    const uint32_t x0 = sw.swap1 ? h.y : h.x, x1 = sw.swap1 ? h.x : h.y;
    const uint32_t x2 = sw.swap1 ? h.w : h.z, x3 = sw.swap1 ? h.z : h.w;
    const uint32_t z[4] = {sw.swap2 ? x2 : x0, sw.swap2 ? x3 : x1, sw.swap2 ? x0 : x2, sw.swap2 ? x1 : x3};
#pragma unroll
    for (int t = 0; t < 16; ++t) {
      const uint32_t off = __builtin_amdgcn_perm(z[t >> 2], sw.mc[qd * 4 + (t >> 2)], sw.sel[t & 3]);
      s += *(const int32_t*)(tbl + off);
    }
  }
  return s;
}

template <int M>
__device__ __forceinline__ int32_t score_exact_row(const uint8_t* row, const unsigned char* tbl,
                                                   const ExactSwizzle<M>& sw) {
  uint4 w[M / 16];
#pragma unroll
  for (int qd = 0; qd < M / 16; ++qd) w[qd] = *(const uint4*)(row + qd * 16);
  return score_exact<M>(w, tbl, sw);
}

// The P0 sampling workgroups of a problem each estimate a head's threshold from their share of the
// sample; the streaming and final kernels use the mean of the estimates (rounded down), which is
// close to what one rank search over the merged sample would give.  INT32_MIN ("take every row")
// from any of them wins.  Exactness never depends on this value: the final kernel proves its
// result complete against whatever threshold was used, or redoes the head exactly.
// Called by all lanes of a wave for NH consecutive heads starting at `head0` (heads at or past
// `n_valid` get 65536, which no coarse score reaches): lane 8 r + p loads part p of head r, so
// the P0 <= 8 values of all heads arrive with one load latency instead of one after another.
// Split in two so that a caller can put its other loads between the request and the use.
template <int NH>
__device__ __forceinline__ int32_t request_thresholds(const int32_t* __restrict__ thr, size_t head0,
                                                      int n_valid, int P0) {
  static_assert(NH * 8 <= 64, "one lane per (head, part)");
  const int lane = threadIdx.x & 63, r = lane >> 3, p = lane & 7;
  int32_t v = 0;
  if (r < NH && r < n_valid && p < P0) v = thr[(head0 + r) * P0 + p];
  return v;
}
template <int NH>
__device__ __forceinline__ void combine_thresholds(int32_t v, int n_valid, int P0, int32_t (&T)[NH]) {
  int32_t all_rows = v == INT32_MIN ? 1 : 0;
  int32_t sum = all_rows ? 0 : v;   // thresholds are >= 0 and below 2^16
  sum = group8_sum(sum);
  all_rows = group8_or(all_rows);
#pragma unroll
  for (int i = 0; i < NH; ++i) {
    const int32_t s_i = __builtin_amdgcn_readlane(sum, 8 * i), a_i = __builtin_amdgcn_readlane(all_rows, 8 * i);
    T[i] = i >= n_valid ? 65536 : (a_i ? INT32_MIN : s_i / P0);
  }
}

// Sum over aligned groups of 16 lanes (one DPP row), result in every lane of the group.
__device__ __forceinline__ int32_t group16_sum(int32_t v) {
  v = group8_sum(v);
  v += __builtin_amdgcn_update_dpp(0, v, 0x140, 0xf, 0xf, false);   // row_mirror
  return v;
}

// Exact score of the token at `row` (its M code bytes) for one head, straight from the head's
// [c][m] table in global memory, by one thread (used for a handful of rows only).
template <int M>
__device__ __forceinline__ int32_t score_exact_global(const uint8_t* __restrict__ row,
                                                      const int32_t* __restrict__ head_table) {
  int32_t s = 0;
#pragma unroll
  for (int qd = 0; qd < M / 16; ++qd) {
    const uint4 w = *(const uint4*)(row + qd * 16);
    const uint32_t ww[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
    for (int t = 0; t < 16; ++t) {
      const uint32_t c = (ww[t >> 2] >> (8 * (t & 3))) & 0xffu;
      s += head_table[c * M + qd * 16 + t];
    }
  }
  return s;
}

// ------------------------------------------------------------------------------------------
// Exact route (also the fallback of the fast route)
// ------------------------------------------------------------------------------------------
struct ExactLds {
  uint32_t hist[kHistBins];
  uint32_t wave_a[kExactThreads / 64];
  uint32_t wave_b[kExactThreads / 64];
  uint32_t res[2];
};

// Exact top-K for one head by the whole workgroup.  `head_table` is the head's [c][m] table in
// global memory, `meta` its four table constants, `tbl` kExactLdsBytes of LDS.  Writes
// out_idx[0..kk) ascending (and out_score); the caller has written the count and the -1 padding.
// Requires sr.kk >= 1.
template <int M>
__device__ void exact_select_block(const uint8_t* __restrict__ seq_codes,
                                   const int32_t* __restrict__ head_table,
                                   const int32_t* __restrict__ meta, float scale,
                                   const SeqRange& sr, int32_t* __restrict__ out_idx,
                                   float* __restrict__ out_score, unsigned char* tbl, ExactLds& L) {
  constexpr int NT = kExactThreads;
  const int tid = threadIdx.x;
  const int32_t s_lo = meta[0], s_hi = meta[2];   // bounds of any score
  ExactSwizzle<M> sw;
  sw.init(tid & 63);
  __syncthreads();   // tbl may alias LDS the caller was still reading
  load_exact_table<M, NT>(head_table, tbl);
  __syncthreads();

  const int lo = sr.sink_end, hi = sr.win_start;
  uint32_t kth = 0, k_rem = (uint32_t)sr.kk;
  if (sr.kk < sr.ncand) {
    // Radix digits are taken from key - key(lower bound of any score), so that the histogram bins
    // spread over the occupied range instead of all keys sharing their leading bits.
    const uint32_t k_lo = score_key(s_lo);
    int remaining = 32 - __clz(score_key(s_hi) - k_lo);   // significant bits of a relative key
    uint32_t prefix = 0, mask = 0;
#pragma unroll 1
    while (remaining > 0) {
      const int bits = remaining < 11 ? remaining : 11;
      const int shift = remaining - bits;
      const uint32_t dmask = (1u << bits) - 1u;
      for (int i = tid; i < kHistBins; i += NT) L.hist[i] = 0;
      __syncthreads();
      for (int j = lo + tid; j < hi; j += NT) {
        const uint32_t key = score_key(score_exact_row<M>(seq_codes + (size_t)j * M, tbl, sw)) - k_lo;
        if ((key & mask) == prefix) atomicAdd(&L.hist[(key >> shift) & dmask], 1u);
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

  // Ordered emission: keys above the K-th, plus the first k_rem positions that equal it.
  uint32_t eq_seen = 0, out_n = 0;
  const bool take_all = sr.kk >= sr.ncand;
#pragma unroll 1
  for (int base = lo; base < hi; base += NT) {
    const int j = base + tid;
    int32_t s = 0;
    uint32_t gt = 0, eq = 0;
    if (j < hi) {
      s = score_exact_row<M>(seq_codes + (size_t)j * M, tbl, sw);
      const uint32_t key = score_key(s);
      gt = take_all ? 1u : (key > kth ? 1u : 0u);
      eq = take_all ? 0u : (key == kth ? 1u : 0u);
    }
    uint32_t tot_eq, tot_sel;
    const uint32_t ex_eq = block_exclusive_scan<NT>(eq, L.wave_a, tot_eq);
    const uint32_t sel = gt | ((eq && (eq_seen + ex_eq < k_rem)) ? 1u : 0u);
    const uint32_t ex_sel = block_exclusive_scan<NT>(sel, L.wave_b, tot_sel);
    if (sel) {
      const uint32_t pos = out_n + ex_sel;
      out_idx[pos] = j;
      if (out_score) out_score[pos] = (float)s * scale;
    }
    eq_seen += tot_eq;
    out_n += tot_sel;
    if (out_n >= (uint32_t)sr.kk) break;
  }
}

template <int M>
__global__ __launch_bounds__(kExactThreads) void select_exact_kernel(
    const uint8_t* __restrict__ codes, const int32_t* __restrict__ lut,
    const float* __restrict__ lut_scale, const int32_t* __restrict__ seq_lens,
    int32_t* __restrict__ topk_idx, int32_t* __restrict__ topk_count,
    float* __restrict__ topk_score, int B, int Hq, int Hkv, int ctx_len, int64_t ctx_stride,
    int top_k, int window, int n_sink) {
  extern __shared__ __align__(16) unsigned char dyn_lds[];
  __shared__ ExactLds L;
  const int bh = blockIdx.x, b = bh / Hq, h = bh % Hq;
  const int G = Hq / Hkv, kv = h / G;
  const SeqRange sr = seq_range(ctx_len, seq_lens, b, window, n_sink, top_k);
  int32_t* oi = topk_idx + (size_t)bh * top_k;
  float* os = topk_score ? topk_score + (size_t)bh * top_k : nullptr;
  if (threadIdx.x == 0) topk_count[bh] = sr.kk;
  for (int t = sr.kk + threadIdx.x; t < top_k; t += kExactThreads) {
    oi[t] = -1;
    if (os) os[t] = 0.f;
  }
  if (sr.kk == 0) return;
  const LutLayout lay = lut_layout(B, Hq, Hkv, M);
  exact_select_block<M>(codes + ((size_t)b * Hkv + kv) * ctx_stride * M,
                        lut + lay.off_exact + (size_t)bh * (kCentroids * M), lut + lay.off_meta + (size_t)bh * 4,
                        lut_scale[bh], sr, oi, os, dyn_lds, L);
}

// ------------------------------------------------------------------------------------------
// Debug: dense exact scores for every token (not on the fast path; used by parity tests)
// ------------------------------------------------------------------------------------------
template <int M>
__global__ __launch_bounds__(kStreamThreads) void score_dense_kernel(
    const uint8_t* __restrict__ codes, const int32_t* __restrict__ lut,
    const float* __restrict__ lut_scale, const int32_t* __restrict__ seq_lens,
    float* __restrict__ scores_out, int B, int Hq, int Hkv, int ctx_len, int64_t ctx_stride) {
  extern __shared__ __align__(16) unsigned char dyn_lds[];
  unsigned char* tbl = dyn_lds;
  const int bh = blockIdx.y, b = bh / Hq, h = bh % Hq;
  const int G = Hq / Hkv, kv = h / G;
  const LutLayout lay = lut_layout(B, Hq, Hkv, M);
  load_exact_table<M, kStreamThreads>(lut + lay.off_exact + (size_t)bh * (kCentroids * M), tbl);
  ExactSwizzle<M> sw;
  sw.init(threadIdx.x & 63);
  __syncthreads();
  int n = seq_lens ? seq_lens[b] : ctx_len;
  n = n < 0 ? 0 : (n > ctx_len ? ctx_len : n);
  const uint8_t* seq_codes = codes + ((size_t)b * Hkv + kv) * ctx_stride * M;
  const float sc = lut_scale[bh];
  for (int j = blockIdx.x * kStreamThreads + threadIdx.x; j < n; j += gridDim.x * kStreamThreads)
    scores_out[(size_t)bh * ctx_stride + j] = (float)score_exact_row<M>(seq_codes + (size_t)j * M, tbl, sw) * sc;
}

// ------------------------------------------------------------------------------------------
// Fast route, stage 1: sampled coarse thresholds
// ------------------------------------------------------------------------------------------
template <int M>
__global__ __launch_bounds__(kSampleThreads) void sample_threshold_kernel(
    const uint8_t* __restrict__ codes, const int32_t* __restrict__ lut,
    const int32_t* __restrict__ seq_lens, int32_t* __restrict__ thr, int B, int Hq, int Hkv, int NG,
    int P0, int sample_rows, int problems, int ctx_len, int64_t ctx_stride, int top_k, int window,
    int n_sink) {
  extern __shared__ __align__(16) unsigned char dyn_lds[];
  int p, prob;
  xcd_map_sets(blockIdx.x, P0, problems, NG, prob, p);
  sample_threshold_body<M, kSampleThreads, false>(prob, p, codes, lut, seq_lens, thr, B, Hq, Hkv, NG, P0, sample_rows,
                                                  ctx_len, ctx_stride, top_k, window, n_sink, dyn_lds);
}

// ------------------------------------------------------------------------------------------
// Fast route, stage 2: one pass over the code matrix
// ------------------------------------------------------------------------------------------
// RESHARED: the rows are read by more than one problem (the head groups of a KV head, placed next
// to each other on one XCD): ordinary loads, so that the line stays in that L2 for the neighbour;
// otherwise non-temporal loads (each row is read once).
//
// A workgroup owns tiles_per_chunk consecutive tiles of one problem; wave w takes every eighth of
// them starting at the w-th, so the eight waves stream one contiguous region together.  A wave
// works in units of 256 rows (4 per lane) with two register sets: both are requested right after
// the workgroup's table copy has been requested (loads return in order, so the table must not
// queue behind cold rows), and each is requested again as soon as it has been consumed, so HBM
// streams from the first microsecond on while the table is still on its way to LDS.
template <int M, bool RESHARED>
__device__ __forceinline__ void stream_select_body(
    const uint8_t* __restrict__ codes, const int32_t* __restrict__ lut,
    const int32_t* __restrict__ seq_lens, const int32_t* __restrict__ thr,
    uint32_t* __restrict__ seg_meta, uint32_t* __restrict__ cand, int B, int Hq, int Hkv, int NG,
    int P0, int n_chunks, int problems, int n_tiles, int tiles_per_chunk, int tile_rows, int row_cap,
    int ctx_len, int64_t ctx_stride, int top_k, int window, int n_sink) {
  constexpr int NT = kStreamThreads;
  constexpr int U = kTileUnit / 64;   // rows per lane and unit
  extern __shared__ __align__(16) unsigned char dyn_lds[];
  unsigned char* tbl = dyn_lds;

  int chunk, prob;
  xcd_map_sets(blockIdx.x, n_chunks, problems, NG, prob, chunk);
  const int g4 = prob % NG, kv = (prob / NG) % Hkv, b = prob / (NG * Hkv);
  const int G = Hq / Hkv, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const SeqRange sr = seq_range(ctx_len, seq_lens, b, window, n_sink, top_k);
  const int t_begin = chunk * tiles_per_chunk, t_end = min(n_tiles, t_begin + tiles_per_chunk);
  const int tsub = tile_rows / kTileUnit;
  uint32_t* meta0 = seg_meta + (size_t)prob * n_tiles * kSegMeta;
  uint32_t* cand0 = cand + (size_t)prob * n_tiles * ((size_t)row_cap * kEntryWords);
  auto tile_row0 = [&](int t) { return (long)sr.sink_end + (long)t * tile_rows; };

  // thresholds of the group's heads: requested here, combined after the table copy has been issued
  const int32_t thr_lane = request_thresholds<4>(thr, (size_t)b * Hq + kv * G + g4 * kHeadsPerGroup,
                                                G - g4 * kHeadsPerGroup, P0);
  int32_t T[4];   // padded heads never want a row
  // This wave's tiles: t_begin + wv, + 8, ...; those that start inside the candidate range are
  // scored (they come first), the others (a sequence shorter than the planned context) only get
  // an empty segment header.
  int my_tiles = 0, n_live = 0;
  for (int t = t_begin + wv; t < t_end; t += kStreamWaves) {
    ++my_tiles;
    if (tile_row0(t) < sr.win_start) ++n_live;
  }
  // The scoring loop addresses the table by absolute LDS address (it must start at 0, which holds
  // because this kernel has no static LDS).  Should a toolchain ever place it elsewhere, publish
  // overflowing segments instead: the final kernel then takes the exact route.
  const bool misplaced = (uint32_t)(uintptr_t)tbl != 0u;
  auto publish_empty = [&](int first) {   // headers of this wave's tiles from its `first`-th on
    for (int i = first; i < my_tiles; ++i)
      if (lane < kSegMeta)
        meta0[(size_t)(t_begin + wv + i * kStreamWaves) * kSegMeta + lane] = misplaced && lane == 0 ? 0xffffffffu : 0u;
  };
  if (tile_row0(t_begin) >= sr.win_start || misplaced) {   // nothing to score in this workgroup (uniform over it)
    publish_empty(0);
    return;
  }

  LaneSwizzle<M> sw;
  sw.init(lane);
  const uint8_t* seq_codes = codes + ((size_t)b * Hkv + kv) * ctx_stride * M;
  const int n_units = n_live * tsub;

  struct Cursor { int t, sub; };
  auto advance = [&](Cursor& c) {
    if (++c.sub == tsub) {
      c.sub = 0;
      c.t += kStreamWaves;
    }
  };
  // Rows of a unit.  Loads are never skipped, also not for a unit past the wave's last one: a load
  // under a branch would make every later wait cover all loads in flight instead of the older
  // register set only.  The row index is clamped into the candidate range (this workgroup has
  // candidates), and rows past the end of a tile are masked out when they are scored.
  uint4 rows_a[U][M / 16], rows_b[U][M / 16];
  auto load_rows = [&](const Cursor& c, uint4 (&dst)[U][M / 16]) {
    const long t0 = min(tile_row0(c.t), (long)sr.win_start - 1);
    const int last = (int)min((long)sr.win_start, t0 + tile_rows) - 1;   // >= t0 >= sink_end
    const int base = (int)t0 + c.sub * kTileUnit;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int j = base + u * 64 + lane;
      const int jl = j < last ? j : last;
#pragma unroll
      for (int qd = 0; qd < M / 16; ++qd)
        dst[u][qd] = load_global_u4<!RESHARED>(seq_codes + (size_t)jl * M + ((uint32_t)(qd * 16) ^ sw.row_swz));
    }
  };

  int n_rows = 0;                  // entries written to the current segment by this wave (wave-uniform)
  int n_head[4] = {0, 0, 0, 0};    // of which wanted by each head
  uint32_t* my_ent = cand0;
  auto process = [&](const Cursor& c, const uint4 (&rows)[U][M / 16]) {
    const long t0 = tile_row0(c.t);
    const int end = (int)min((long)sr.win_start, t0 + tile_rows);
    const int base = (int)t0 + c.sub * kTileUnit;
    if (c.sub == 0) {   // (wave-uniform) a new tile: a new segment
      n_rows = 0;
#pragma unroll
      for (int r = 0; r < 4; ++r) n_head[r] = 0;
      my_ent = cand0 + (size_t)c.t * ((size_t)row_cap * kEntryWords);
    }
    // Scores and the per-head "reaches the threshold" wave masks are formed together, so the
    // gathered table entries die inside this straight-line block.  The masks live in scalar
    // registers; their popcounts cost no vector instructions.
    uint64_t hit[U][4];
    uint32_t a01[U], a23[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      score_coarse<M, true>(rows[u], tbl, sw, a01[u], a23[u]);
      const uint64_t valid = __builtin_amdgcn_ballot_w64(base + u * 64 + lane < end);
      hit[u][0] = __builtin_amdgcn_ballot_w64((int32_t)(a01[u] & 0xffffu) >= T[0]) & valid;
      hit[u][1] = __builtin_amdgcn_ballot_w64((int32_t)(a01[u] >> 16) >= T[1]) & valid;
      hit[u][2] = __builtin_amdgcn_ballot_w64((int32_t)(a23[u] & 0xffffu) >= T[2]) & valid;
      hit[u][3] = __builtin_amdgcn_ballot_w64((int32_t)(a23[u] >> 16) >= T[3]) & valid;
      if (u & 1) __builtin_amdgcn_sched_barrier(0);   // two rows' gathers at a time: bounds live registers
    }
    // A surviving row is written once: position and the coarse scores of the four heads (the final
    // kernel of a head tells from them whether the head wants the row).  Slots come from the lane
    // masks: no atomics, and the entries of a segment are in ascending position.
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const uint64_t any = hit[u][0] | hit[u][1] | hit[u][2] | hit[u][3];
      if (any) {
        if (__builtin_amdgcn_inverse_ballot_w64(any)) {
          const int slot = (int)__builtin_amdgcn_mbcnt_hi(
              (uint32_t)(any >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)any, (uint32_t)n_rows));
          if (slot < row_cap) {   // rows past the capacity are dropped but still counted
            uint32_t* e = my_ent + (size_t)slot * kEntryWords;
            e[0] = (uint32_t)(base + u * 64 + lane);
            e[1] = a01[u];
            e[2] = a23[u];
          }
        }
        n_rows += __popcll(any);
#pragma unroll
        for (int r = 0; r < 4; ++r) n_head[r] += __popcll(hit[u][r]);
      }
    }
    if (c.sub == tsub - 1 && lane < kSegMeta) {   // header of the tile's segment: entries written, rows per head
      uint32_t v = 0;
      if (lane == 0) v = (uint32_t)n_rows;
#pragma unroll
      for (int r = 0; r < 4; ++r)
        if (lane == 1 + r) v = (uint32_t)n_head[r];
      meta0[(size_t)c.t * kSegMeta + lane] = v;
    }
  };

  // The table copy is requested first, then the first two units of rows; the table is put into
  // LDS as soon as it has arrived (the rows, requested later, are still in flight then).
  constexpr int TPT = kCentroids * M / 2 / NT;   // 16-byte pieces of the table per thread
  int4 tv[TPT];
  {
    const LutLayout lay = lut_layout(B, Hq, Hkv, M);
    const int4* src = (const int4*)(lut + lay.off_coarse + (size_t)prob * (kCentroids * M * 2));
    // Both pointers pass through an empty asm, so the compiler no longer knows that they point to
    // read-only, unaliased memory and keeps the table loads, the asm below and the row loads in
    // this order (it otherwise issues the row loads first).
    asm volatile("" : "+s"(src));
    asm volatile("" : "+s"(seq_codes));
#pragma unroll
    for (int k = 0; k < TPT; ++k) {
      const uint4 v = load_global_u4<false>(src + tid + k * NT);
      tv[k] = make_int4((int)v.x, (int)v.y, (int)v.z, (int)v.w);
    }
  }
  asm volatile("" ::: "memory");
  __builtin_amdgcn_sched_barrier(0);
  Cursor ld{t_begin + wv, 0}, pr{t_begin + wv, 0};
  load_rows(ld, rows_a);
  advance(ld);
  load_rows(ld, rows_b);
  advance(ld);
#pragma unroll
  for (int k = 0; k < TPT; ++k) {
    const int e = tid + k * NT;   // pair of entries (2 e, 2 e + 1) of the global order [half][c][16 m]
    const int half = e / (kCentroids * 8), c = (e / 8) % kCentroids, mp = e % 8;
    store_coarse_lds<M>(tbl, c, 16 * half + 2 * mp, tv[k]);
  }
  combine_thresholds<4>(thr_lane, G - g4 * kHeadsPerGroup, P0, T);
  __syncthreads();   // (every wave of the workgroup gets here, also one without live tiles)
#pragma unroll 1
  for (int v = 0; v < n_units; v += 2) {
    process(pr, rows_a);
    advance(pr);
    load_rows(ld, rows_a);
    advance(ld);
    if (v + 1 < n_units) {
      process(pr, rows_b);
      advance(pr);
    }
    load_rows(ld, rows_b);
    advance(ld);
  }
  publish_empty(n_live);
}

#define A2ATS_STREAM_ARGS                                                                          \
  const uint8_t *__restrict__ codes, const int32_t *__restrict__ lut,                             \
      const int32_t *__restrict__ seq_lens, const int32_t *__restrict__ thr,                      \
      uint32_t *__restrict__ seg_meta, uint32_t *__restrict__ cand, int B, int Hq, int Hkv, int NG,  \
      int P0, int n_chunks, int problems, int n_tiles, int tiles_per_chunk, int tile_rows,         \
      int row_cap, int ctx_len, int64_t ctx_stride, int top_k, int window, int n_sink
#define A2ATS_STREAM_PASS                                                                          \
  codes, lut, seq_lens, thr, seg_meta, cand, B, Hq, Hkv, NG, P0, n_chunks, problems, n_tiles,      \
      tiles_per_chunk, tile_rows, row_cap, ctx_len, ctx_stride, top_k, window, n_sink

// 64 KB of LDS per workgroup.  M = 16: 128 VGPRs -> 4 waves per SIMD (two workgroups per CU).
__global__ __launch_bounds__(kStreamThreads) __attribute__((amdgpu_waves_per_eu(4, 4)))
void stream_select_kernel16(A2ATS_STREAM_ARGS) { stream_select_body<16, false>(A2ATS_STREAM_PASS); }
__global__ __launch_bounds__(kStreamThreads) __attribute__((amdgpu_waves_per_eu(4, 4)))
void stream_select_kernel16r(A2ATS_STREAM_ARGS) { stream_select_body<16, true>(A2ATS_STREAM_PASS); }
// M = 32: twice the row registers.
__global__ __launch_bounds__(kStreamThreads) __attribute__((amdgpu_waves_per_eu(2, 4)))
void stream_select_kernel32(A2ATS_STREAM_ARGS) { stream_select_body<32, false>(A2ATS_STREAM_PASS); }
__global__ __launch_bounds__(kStreamThreads) __attribute__((amdgpu_waves_per_eu(2, 4)))
void stream_select_kernel32r(A2ATS_STREAM_ARGS) { stream_select_body<32, true>(A2ATS_STREAM_PASS); }

// ------------------------------------------------------------------------------------------
// Fast route, stage 3: the K-th coarse score, exact ranking of the rows around it, ordered output
// ------------------------------------------------------------------------------------------
// Route words (diagnostics): 0 fast; 1 fewer survivors than K; 2 more than the LDS list holds;
// 3 a segment overflowed; 4 the threshold is not far enough below the K-th coarse score for the
// list to be complete; 5 more than kBandMax rows within M coarse units of the K-th coarse score.
// 1..5 end in the exact route for that head.
template <int M>
__global__ __launch_bounds__(kExactThreads) void final_select_kernel(
    const uint8_t* __restrict__ codes, const int32_t* __restrict__ lut,
    const float* __restrict__ lut_scale, const int32_t* __restrict__ seq_lens,
    const int32_t* __restrict__ thr, const uint32_t* __restrict__ seg_meta,
    const uint32_t* __restrict__ cand, uint32_t* __restrict__ route, int32_t* __restrict__ topk_idx,
    int32_t* __restrict__ topk_count, float* __restrict__ topk_score, int B, int Hq, int Hkv, int NG,
    int P0, int problems, int n_seg, int row_cap, int cap, int ctx_len, int64_t ctx_stride, int top_k,
    int window, int n_sink) {
  constexpr int NT = kExactThreads;
  extern __shared__ __align__(16) unsigned char dyn_lds[];
  __shared__ ExactLds L;
  __shared__ uint32_t s_seg_off[kMaxTiles + 1];
  __shared__ uint16_t s_seg_rows[kMaxTiles];
  __shared__ uint16_t s_band_idx[kBandMax];
  __shared__ uint32_t s_sub[32];
  __shared__ uint32_t s_overflow, s_n_band, s_n_sure, s_ck, s_ngt;

  // one workgroup per (problem, head slot), on the XCD that streamed the problem
  int prob, r;
  xcd_map_sets(blockIdx.x, kHeadsPerGroup, problems, NG, prob, r);
  const int G = Hq / Hkv;
  const int g4 = prob % NG, kv = (prob / NG) % Hkv, b = prob / (NG * Hkv);
  const int hg = g4 * kHeadsPerGroup + r;
  if (hg >= G) return;
  const int bh = b * Hq + kv * G + hg, tid = threadIdx.x, lane = tid & 63;
  const SeqRange sr = seq_range(ctx_len, seq_lens, b, window, n_sink, top_k);
  int32_t* oi = topk_idx + (size_t)bh * top_k;
  float* os = topk_score ? topk_score + (size_t)bh * top_k : nullptr;
  if (tid == 0) topk_count[bh] = sr.kk;
  for (int t = sr.kk + tid; t < top_k; t += NT) {
    oi[t] = -1;
    if (os) os[t] = 0.f;
  }
  if (sr.kk == 0) {
    if (tid == 0) route[bh] = 0u;
    return;
  }
  const float scale = lut_scale[bh];
  const LutLayout lay = lut_layout(B, Hq, Hkv, M);
  const int32_t* head_table = lut + lay.off_exact + (size_t)bh * (kCentroids * M);
  const int32_t* meta = lut + lay.off_meta + (size_t)bh * 4;
  const uint8_t* seq_codes = codes + ((size_t)b * Hkv + kv) * ctx_stride * M;

  // LDS: the head's survivors in position order -- coarse score (bit 17: winner) and position.
  // (The exact route, if it comes to that, puts the head's table over them.)
  uint32_t* c_key = (uint32_t*)dyn_lds;
  uint32_t* c_pos = c_key + cap;

  // Segment headers of the problem (one per tile of the streaming pass) and the head's threshold.
  uint32_t seg_rows = 0, my_cnt = 0;
  if (tid < n_seg) {
    const uint32_t* mt = seg_meta + ((size_t)prob * n_seg + tid) * kSegMeta;
    seg_rows = mt[0];
    my_cnt = mt[1 + r];
  }
  const int32_t thr_lane = request_thresholds<1>(thr, (size_t)bh, 1, P0);
  int32_t tc1[1];
  combine_thresholds<1>(thr_lane, 1, P0, tc1);
  const int32_t tc = tc1[0];
  for (int i = tid; i < kHistBins; i += NT) L.hist[i] = 0;
  if (tid < 32) s_sub[tid] = 0;
  if (tid == 0) {
    s_overflow = 0;
    s_n_band = 0;
    s_n_sure = 0;
  }
  __syncthreads();
  if (tid < n_seg) {
    if (seg_rows > (uint32_t)row_cap) s_overflow = 1;
    s_seg_rows[tid] = (uint16_t)min(seg_rows, 65535u);
  }
  uint32_t n_c;   // rows this head wants, over all segments
  const uint32_t my_off = block_exclusive_scan<NT>(my_cnt, L.wave_a, n_c);
  if (tid < n_seg) s_seg_off[tid] = my_off;
  __syncthreads();
  if (s_overflow || n_c > (uint32_t)cap || n_c < (uint32_t)sr.kk) {
    if (tid == 0) route[bh] = s_overflow ? 3u : (n_c > (uint32_t)cap ? 2u : 1u);
    exact_select_block<M>(seq_codes, head_table, meta, scale, sr, oi, os, dyn_lds, L);
    return;
  }

  // Every row the head wants has a coarse score in [lo, 65535]; the first histogram level spreads
  // its 2048 bins over that range (bins of 2^shift1 <= 32 values).
  const uint32_t lo = tc == INT32_MIN ? 0u : (uint32_t)min(max(tc, 0), 65535);
  const int nbits = 32 - __clz(65535u - lo);
  const int bits1 = nbits < 11 ? nbits : 11, shift1 = nbits - bits1;
  {
    // Pass 1: the rows this head wants, out of the problem's entries, into LDS in position order.
    // A group of tps lanes (a power of two, inside one wave) shares a segment and walks its
    // entries tps at a time; destination = head's rows in earlier segments + rows the group has
    // passed + rank among the lanes of this step (a ballot), so no thread waits for another.
    int tps = 64;
    while (tps > 1 && tps * n_seg > NT) tps >>= 1;   // n_seg <= 512: at least 2
    const int g = tid / tps, pl = tid % tps;
    const bool act = g < n_seg;
    const uint32_t n_rows = act ? (uint32_t)s_seg_rows[g] : 0u, dst0 = act ? s_seg_off[g] : 0u;
    const uint32_t max_rows = (uint32_t)__builtin_amdgcn_readlane((int)wave_max_to_last_lane(n_rows), 63);
    const uint32_t* ent = cand + ((size_t)prob * n_seg + (act ? g : 0)) * ((size_t)row_cap * kEntryWords);
    const int gshift = (lane / tps) * tps;
    const uint64_t gmask = (tps == 64 ? ~0ull : ((1ull << tps) - 1ull)) << gshift;
    const uint64_t below = gmask & ((1ull << lane) - 1ull);
    constexpr int kInFlight = 4;
    uint32_t running = 0;
    for (uint32_t i0 = 0; i0 < max_rows; i0 += kInFlight * tps) {
      uint32_t e_pos[kInFlight], e_w[kInFlight];
#pragma unroll
      for (int k = 0; k < kInFlight; ++k) {
        const uint32_t i = i0 + k * tps + pl;
        e_pos[k] = 0;
        e_w[k] = 0;
        if (i < n_rows) {
          const uint32_t* e = ent + (size_t)i * kEntryWords;
          e_pos[k] = e[0];
          e_w[k] = e[1 + (r >> 1)];
        }
      }
#pragma unroll
      for (int k = 0; k < kInFlight; ++k) {
        const uint32_t i = i0 + k * tps + pl;
        const uint32_t coarse = (r & 1) ? (e_w[k] >> 16) : (e_w[k] & 0xffffu);
        const bool wanted = i < n_rows && (int32_t)coarse >= tc;
        const uint64_t m = __builtin_amdgcn_ballot_w64(wanted);
        if (wanted) {
          const uint32_t dst = dst0 + running + (uint32_t)__popcll(m & below);
          if (dst < n_c) {   // always true for a consistent workspace; keeps LDS writes in range whatever it holds
            c_pos[dst] = e_pos[k];
            c_key[dst] = coarse;
            atomicAdd(&L.hist[min((coarse - lo) >> shift1, (uint32_t)kHistBins - 1)], 1u);
          }
        }
        running += (uint32_t)__popcll(m & gmask);
      }
    }
  }
  __syncthreads();

  // The K-th largest coarse score c_K and the number of rows above it: first level by bins, then
  // the values inside the K-th row's bin (at most 32).
  block_find_rank_desc<NT, kHistBins>([&](int i) { return L.hist[i]; }, (uint32_t)sr.kk, L.wave_a, L.res);
  const uint32_t bin1 = L.res[0], above1 = L.res[1];
  uint32_t c_k, n_gt;
  if (shift1 == 0) {
    c_k = lo + bin1;
    n_gt = above1;
  } else {
    const uint32_t nsub = 1u << shift1, smask = nsub - 1u;
    for (uint32_t i = tid; i < n_c; i += NT) {
      const uint32_t rel = c_key[i] - lo;
      if ((rel >> shift1) == bin1) atomicAdd(&s_sub[rel & smask], 1u);
    }
    __syncthreads();
    if (tid < 64) {   // lane l < nsub looks at value nsub - 1 - l of the bin (values descend with the lane)
      const uint32_t v = (uint32_t)lane < nsub ? s_sub[nsub - 1u - lane] : 0u;
      const uint32_t incl = wave_inclusive_scan(v);
      const uint64_t reach = __builtin_amdgcn_ballot_w64((uint32_t)lane < nsub && above1 + incl >= (uint32_t)sr.kk);
      const int l0 = reach ? __ffsll((unsigned long long)reach) - 1 : 0;
      if (lane == l0) {
        s_ck = lo + (bin1 << shift1) + (nsub - 1u - (uint32_t)l0);
        s_ngt = above1 + incl - v;
      }
    }
    __syncthreads();
    c_k = s_ck;
    n_gt = s_ngt;
  }
  (void)n_gt;

  // Completeness: every row with coarse score above c_K - M must be on the list, i.e. the
  // threshold (a row is listed iff its coarse score reaches it) must not exceed c_K - M + 1.
  if (tc != INT32_MIN && (long)c_k < (long)tc + M - 1) {
    if (tid == 0) route[bh] = 4u;
    exact_select_block<M>(seq_codes, head_table, meta, scale, sr, oi, os, dyn_lds, L);
    return;
  }

  // Classes: coarse >= c_K + M wins (bit 17); c_K - M < coarse < c_K + M is decided below by exact
  // scores; anything else loses.  Counts and band slots are aggregated per wave.
  for (uint32_t i0 = 0; i0 < n_c; i0 += NT) {
    const uint32_t i = i0 + tid;
    const uint32_t key = i < n_c ? c_key[i] : 0u;
    const bool sure = i < n_c && key >= c_k + (uint32_t)M;
    const bool band = i < n_c && !sure && key + (uint32_t)M > c_k;
    const uint64_t ms = __builtin_amdgcn_ballot_w64(sure), mb = __builtin_amdgcn_ballot_w64(band);
    uint32_t base_b = 0;
    if (lane == 0) {
      if (ms) atomicAdd(&s_n_sure, (uint32_t)__popcll(ms));
      if (mb) base_b = atomicAdd(&s_n_band, (uint32_t)__popcll(mb));
    }
    base_b = (uint32_t)__builtin_amdgcn_readfirstlane((int)base_b);
    if (sure) c_key[i] = key | 0x20000u;
    if (band) {
      const uint32_t j = base_b + (uint32_t)lanes_below(mb);
      if (j < (uint32_t)kBandMax) s_band_idx[j] = (uint16_t)i;
    }
  }
  __syncthreads();
  const uint32_t n_band = s_n_band, n_sure = s_n_sure;
  if (n_band > (uint32_t)kBandMax) {
    if (tid == 0) route[bh] = 5u;
    exact_select_block<M>(seq_codes, head_table, meta, scale, sr, oi, os, dyn_lds, L);
    return;
  }
  if (tid == 0) route[bh] = 0u;
  // At most K - 1 rows have a coarse score above c_K, so fewer than K are sure winners, and at
  // least K reach c_K, so the band holds the rest.
  const uint32_t k_need = (uint32_t)sr.kk - n_sure;

  // Exact scores of the band rows: 16 lanes per row, each adds the entries of M / 16 subspaces
  // (code bytes from the code matrix, entries from the head's table in global memory), summed
  // over the 16 lanes.  Keys and positions go where the histogram was.
  uint32_t* b_key = L.hist;
  uint32_t* b_pos = L.hist + kBandMax;
  for (uint32_t b0 = 0; b0 < n_band; b0 += NT / 16) {
    const uint32_t bi = b0 + (uint32_t)tid / 16u, l16 = (uint32_t)tid & 15u;
    int32_t e = 0;
    uint32_t pos = 0;
    if (bi < n_band) {
      pos = c_pos[s_band_idx[bi]];
      const uint8_t* row = seq_codes + (size_t)pos * M;
#pragma unroll
      for (int qd = 0; qd < M / 16; ++qd) {
        const uint32_t m = l16 + 16u * qd;
        e += head_table[(uint32_t)row[m] * M + m];
      }
    }
    e = group16_sum(e);
    if (bi < n_band && l16 == 0) {
      b_key[bi] = score_key(e);
      b_pos[bi] = pos;
    }
  }
  __syncthreads();
  // Rank inside the band: a row wins iff fewer than k_need band rows beat it (higher exact score,
  // or the same score at a lower position).
  for (uint32_t bi = tid; bi < n_band; bi += NT) {
    const uint32_t key = b_key[bi], pos = b_pos[bi];
    uint32_t beat = 0;
    for (uint32_t j = 0; j < n_band; ++j) {
      const uint32_t kj = b_key[j];
      beat += (kj > key || (kj == key && b_pos[j] < pos)) ? 1u : 0u;
    }
    if (beat < k_need) c_key[s_band_idx[bi]] |= 0x20000u;
  }
  __syncthreads();

  // Winners in ascending position: the list is sorted by position, so a winner's output slot is
  // the number of winners before it (one block scan over per-thread counts of a contiguous run).
  const uint32_t per = (n_c + NT - 1) / NT;
  const uint32_t i0 = min(n_c, (uint32_t)tid * per), i1 = min(n_c, i0 + per);
  uint32_t loc = 0;
  for (uint32_t i = i0; i < i1; ++i) loc += (c_key[i] >> 17) & 1u;
  uint32_t tot;
  uint32_t slot = block_exclusive_scan<NT>(loc, L.wave_b, tot);
  for (uint32_t i = i0; i < i1; ++i) {
    if ((c_key[i] >> 17) & 1u) {
      const uint32_t pos = c_pos[i];
      if (slot < (uint32_t)sr.kk) {
        oi[slot] = (int32_t)pos;
        if (os) os[slot] = (float)score_exact_global<M>(seq_codes + (size_t)pos * M, head_table) * scale;
      }
      ++slot;
    }
  }
}

// ------------------------------------------------------------------------------------------
// Host side
// ------------------------------------------------------------------------------------------
__global__ void fill_words_kernel(uint32_t* __restrict__ out, uint32_t value, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) out[i] = value;
}

__global__ void sum_segments_kernel(const uint32_t* __restrict__ seg_meta, const uint32_t* __restrict__ route,
                                    uint32_t* __restrict__ out, int B, int Hq, int Hkv, int NG, int n_seg) {
  const int bh = blockIdx.x * blockDim.x + threadIdx.x;
  if (bh >= B * Hq) return;
  const int G = Hq / Hkv, b = bh / Hq, h = bh % Hq, kv = h / G, hg = h % G;
  const size_t prob = ((size_t)b * Hkv + kv) * NG + hg / kHeadsPerGroup;
  uint32_t tot = 0;
  for (int s = 0; s < n_seg; ++s) tot += seg_meta[(prob * n_seg + s) * kSegMeta + 1 + (hg % kHeadsPerGroup)];
  out[bh] = min(tot, 0x0fffffffu) | (route[bh] << 28);
}

hipError_t copy_topk_stats(const a2ats_dims& d, int top_k, int window, int n_sink, const void* ws,
                           uint32_t* cand_counts, hipStream_t stream) {
  const TopkPlan plan = make_topk_plan(d, top_k, window, n_sink);
  const int heads = d.batch * d.n_q_heads;
  if (heads == 0) return hipSuccess;
  if (!plan.fast) {   // (a fill kernel, not a memset node: the call may be captured into a graph)
    hipLaunchKernelGGL(fill_words_kernel, dim3((heads + 255) / 256), dim3(256), 0, stream, cand_counts, 0xffffffffu,
                       heads);
    return hipGetLastError();
  }
  hipLaunchKernelGGL(sum_segments_kernel, dim3((heads + 255) / 256), dim3(256), 0, stream,
                     (const uint32_t*)((const unsigned char*)ws + plan.off_count),
                     (const uint32_t*)((const unsigned char*)ws + plan.off_route), cand_counts, d.batch,
                     d.n_q_heads, d.n_kv_heads, plan.NG, plan.n_tiles);
  return hipGetLastError();
}

template <int M>
static hipError_t launch_score_topk_m(const a2ats_dims& d, const TopkPlan& plan, const uint8_t* codes,
                                      const int32_t* lut, const float* lut_scale, int top_k, int window,
                                      int n_sink, const int32_t* seq_lens, int32_t* topk_idx,
                                      int32_t* topk_count, float* topk_score, float* scores_out,
                                      void* ws, bool presampled, hipStream_t stream, hipEvent_t ev_start,
                                      hipEvent_t ev_stop) {
  const int B = d.batch, Hq = d.n_q_heads, Hkv = d.n_kv_heads, NG = plan.NG;
  const int heads = B * Hq, problems = B * Hkv * NG;
  const size_t coarse_bytes = (size_t)kCoarseLdsBytes;
  const size_t lut1_bytes = kExactLdsBytes;
  hipError_t err;
  static LdsSlot s_dense[16], s_exact[16], s_sample[16], s_stream[16], s_stream_r[16], s_final[16];
  if (heads == 0) return hipSuccess;

  if (scores_out) {
    if ((err = allow_dynamic_lds(score_dense_kernel<M>, lut1_bytes, s_dense)) != hipSuccess) return err;
    int gx = (d.ctx_len + kStreamThreads * 8 - 1) / (kStreamThreads * 8);
    gx = gx < 1 ? 1 : gx;
    hipLaunchKernelGGL((score_dense_kernel<M>), dim3(gx, heads), dim3(kStreamThreads), lut1_bytes, stream,
                       codes, lut, lut_scale, seq_lens, scores_out, B, Hq, Hkv, d.ctx_len, d.ctx_stride);
    if ((err = hipGetLastError()) != hipSuccess) return err;
  }

  if (!plan.fast) {
    if ((err = allow_dynamic_lds(select_exact_kernel<M>, lut1_bytes, s_exact)) != hipSuccess) return err;
    hipLaunchKernelGGL((select_exact_kernel<M>), dim3(heads), dim3(kExactThreads), lut1_bytes, stream,
                       codes, lut, lut_scale, seq_lens, topk_idx, topk_count, topk_score, B, Hq, Hkv,
                       d.ctx_len, d.ctx_stride, top_k, window, n_sink);
    return hipGetLastError();
  }

  unsigned char* wsb = (unsigned char*)ws;
  int32_t* thr = (int32_t*)(wsb + plan.off_thr);
  uint32_t* seg_meta = (uint32_t*)(wsb + plan.off_count);
  uint32_t* route = (uint32_t*)(wsb + plan.off_route);
  uint32_t* cand = (uint32_t*)(wsb + plan.off_cand);

  if (!presampled) {   // (the fused decode launch has written the thresholds already)
    if ((err = allow_dynamic_lds(sample_threshold_kernel<M>, coarse_bytes, s_sample)) != hipSuccess) return err;
    hipLaunchKernelGGL((sample_threshold_kernel<M>), dim3(plan.P0 * problems), dim3(kSampleThreads),
                       coarse_bytes, stream, codes, lut, seq_lens, thr, B, Hq, Hkv, NG, plan.P0, plan.sample_rows,
                       problems, d.ctx_len, d.ctx_stride, top_k, window, n_sink);
    if ((err = hipGetLastError()) != hipSuccess) return err;
  }

  auto stream_kernel = M == 16 ? (NG > 1 ? stream_select_kernel16r : stream_select_kernel16)
                               : (NG > 1 ? stream_select_kernel32r : stream_select_kernel32);
  if ((err = allow_dynamic_lds(stream_kernel, coarse_bytes, NG > 1 ? s_stream_r : s_stream)) != hipSuccess) return err;
  if (ev_start && ev_stop) {
    // events attached to the dispatch itself: their difference is the kernel's own duration
    hipExtLaunchKernelGGL(stream_kernel, dim3(plan.chunks * problems), dim3(kStreamThreads), coarse_bytes,
                          stream, ev_start, ev_stop, 0, codes, lut, seq_lens, thr, seg_meta, cand, B, Hq,
                          Hkv, NG, plan.P0, plan.chunks, problems, plan.n_tiles, plan.tiles_per_chunk,
                          plan.tile_rows, plan.row_cap, d.ctx_len, d.ctx_stride, top_k, window, n_sink);
  } else {
    hipLaunchKernelGGL(stream_kernel, dim3(plan.chunks * problems), dim3(kStreamThreads), coarse_bytes,
                       stream, codes, lut, seq_lens, thr, seg_meta, cand, B, Hq, Hkv, NG, plan.P0,
                       plan.chunks, problems, plan.n_tiles, plan.tiles_per_chunk, plan.tile_rows,
                       plan.row_cap, d.ctx_len, d.ctx_stride, top_k, window, n_sink);
  }
  if ((err = hipGetLastError()) != hipSuccess) return err;

  const size_t final_lds = std::max(lut1_bytes, (size_t)plan.cap * 8);
  if ((err = allow_dynamic_lds(final_select_kernel<M>, final_lds, s_final)) != hipSuccess) return err;
  hipLaunchKernelGGL((final_select_kernel<M>), dim3(problems * kHeadsPerGroup), dim3(kExactThreads),
                     final_lds, stream, codes, lut, lut_scale, seq_lens, thr, seg_meta, cand, route, topk_idx,
                     topk_count, topk_score, B, Hq, Hkv, NG, plan.P0, problems, plan.n_tiles, plan.row_cap,
                     plan.cap, d.ctx_len, d.ctx_stride, top_k, window, n_sink);
  return hipGetLastError();
}

hipError_t launch_score_topk(const a2ats_dims& d, const uint8_t* codes, const int32_t* lut,
                             const float* lut_scale, int top_k, int window, int n_sink,
                             const int32_t* seq_lens, int32_t* topk_idx, int32_t* topk_count,
                             float* topk_score, float* scores_out, void* ws, bool presampled,
                             hipStream_t stream, hipEvent_t ev_start, hipEvent_t ev_stop) {
  const TopkPlan plan = make_topk_plan(d, top_k, window, n_sink);
  if (d.n_sub == 16)
    return launch_score_topk_m<16>(d, plan, codes, lut, lut_scale, top_k, window, n_sink, seq_lens,
                                   topk_idx, topk_count, topk_score, scores_out, ws, presampled, stream,
                                   ev_start, ev_stop);
  return launch_score_topk_m<32>(d, plan, codes, lut, lut_scale, top_k, window, n_sink, seq_lens,
                                 topk_idx, topk_count, topk_score, scores_out, ws, presampled, stream,
                                 ev_start, ev_stop);
}

}  // namespace a2ats
