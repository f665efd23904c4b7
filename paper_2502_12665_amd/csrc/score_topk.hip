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
//  coarse copy of the tables, and only the survivors are scored exactly.
//    1. sample_threshold_kernel scores a sample of each sequence (about 1/8 of it, taken in
//       128-byte runs spread evenly over the candidates) with the coarse tables and derives, per
//       head, a coarse threshold below the K-th score with a 5-sigma margin (distribution-free
//       for independent rows: it only uses ranks of the sample).
//    2. stream_select_kernel streams all code rows: one 8-byte LDS read per code byte serves the
//       four heads of a group (two heads per 32-bit word, 16 bits each, so one integer add
//       accumulates two heads).  A row whose coarse score reaches the threshold of any of the
//       heads is written once -- a 4-byte header (position, wanting heads) and its code bytes --
//       to the segment of its (problem, chunk, wave) in HBM, in row order.
//    3. final_select_kernel (one workgroup per head) collects its head's survivors (about 1.5 K),
//       scores them exactly from the head's 32-bit table, radix-selects the exact K-th key among
//       them, proves that no row outside the survivor list can reach that key (coarse and exact
//       scores differ by less than M coarse units), and writes the winners in ascending
//       position.  If the proof fails or a list is too short / too long / overflowed -- the
//       sample misled (about 1e-6 per head for independent rows, more when similar rows come in
//       runs) or the input is degenerate -- the workgroup runs the exact route for its head, so
//       the result is always exact with respect to the 32-bit scores.
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
constexpr int kSampleRows = 1024;    // smallest sample of a problem; a sampling workgroup scores up to 8 of these
constexpr int kSmallList = 1024;     // members of the K-th key's bin ranked by brute force

TopkPlan make_topk_plan(const a2ats_dims& d, int top_k, int window, int n_sink) {
  TopkPlan p{};
  const int G = d.n_q_heads / d.n_kv_heads;
  p.NG = (G + kHeadsPerGroup - 1) / kHeadsPerGroup;
  long ncand = (long)d.ctx_len - window - n_sink;
  if (ncand < 0) ncand = 0;
  p.cap = 8192;
  p.fast = !single_codebook(d) && ncand >= 16384 && top_k >= 1 && top_k <= 2048 && 4L * top_k <= ncand;
  if (p.fast) {
    // Sample an eighth of the candidates (at most 65536 rows; in units of 512 rows, at least
    // kSampleRows), shared by at most 8 workgroups of at most 8192 rows each.  The survivors the
    // streaming pass writes and the final kernel reads back shrink with the sample (1.95 K per head
    // at a sixteenth, 1.6 K at an eighth), and sampled rows are cheap while few workgroups carry
    // them: every sampling workgroup pays for a table copy (or, in the fused decode prologue, for
    // the table build) whatever it samples.  So the number of parts is what keeps the sampling
    // launch in one round of the 256 CUs beside the workgroups that encode a one-key append
    // (batch * n_kv_heads * M / 16), with about 2048 rows per part where that leaves a choice; a
    // batch whose problems alone exceed one round (the sampling is then a launch of its own) takes
    // parts of up to 4096 rows.  Measured steps (one-key append, 1/16 in 1024-row parts before):
    // batch 4 x 131072 tokens 82.4 -> 81.3 us, batch 16 x 32768 tokens 122.2 -> 117.6 us, batch 32 x
    // 65536 tokens with 7 heads per KV head 390.7 -> 382.5 us.
    long s_tot = ncand / 8 / 512 * 512;
    if (s_tot < kSampleRows) s_tot = kSampleRows;
    if (s_tot > 64 * kSampleRows) s_tot = 64 * kSampleRows;
    const long problems = (long)d.batch * d.n_kv_heads * p.NG;
    const long enc = ((long)d.batch * d.n_kv_heads * d.n_sub + 15) / 16;
    const long fit = problems > 0 ? (256 - enc) / problems : 8;   // parts per problem that fit one round
    long parts;
    if (fit >= 1) parts = std::min<long>(std::min<long>(8, fit), (s_tot + 2047) / 2048);
    else parts = std::min<long>(8, (s_tot + 4095) / 4096);
    if (parts < 1) parts = 1;
    long rows = s_tot / parts / 512 * 512;
    if (rows < 512) rows = 512;
    if (rows > 8 * kSampleRows) rows = 8 * kSampleRows;
    p.P0 = (int)parts;
    s_tot = rows * parts;
    p.sample_rows = (int)(s_tot / p.P0);   // at most 8192: the histogram counts are 16 bits wide
    long chunks = (512 + problems - 1) / problems;
    const long max_chunks = (ncand + 2047) / 2048;
    if (chunks > max_chunks) chunks = max_chunks;
    if (chunks < 1) chunks = 1;
    if (chunks > 64) chunks = 64;
    // Survivor segments, one per (problem, chunk, wave): a header and row_cap row entries each.
    // The sampling rule (rank r with r - 5 sqrt(r) >= K S / N, plus one per part) lets about
    // r N / S rows per head through -- for small K much more than K -- and a row survives if any of
    // the (up to) four heads wants it.  row_cap is twice that share of a wave's rows plus 16
    // standard deviations of a Poisson count: survivors that come in runs (neighbouring tokens with
    // similar scores) scatter far more between segments than independent ones.  The final kernel
    // handles at most 512 segments per problem, i.e. 64 chunks.
    const double r0 = (double)top_k * (double)s_tot / (double)ncand;
    const double xr = 0.5 * (kSigma + std::sqrt(kSigma * kSigma + 4.0 * r0));
    const double survivors = (xr * xr + 2.0 * p.P0) / (double)s_tot * (double)ncand * 1.25;
    const double keep = std::min(1.0, 4.0 * survivors / (double)ncand);
    long rpc = (ncand + chunks - 1) / chunks;
    rpc = (rpc + kStreamThreads - 1) / kStreamThreads * kStreamThreads;
    const long rows_per_wave = rpc / kStreamWaves;   // a multiple of 64
    const double mu = rows_per_wave * keep;
    long cap_rows = (long)(mu * 2.0 + 16.0 * std::sqrt(mu)) + 64;   // generous: unused capacity costs only scratch
    cap_rows = (cap_rows + 31) / 32 * 32;
    if (cap_rows > rows_per_wave) cap_rows = rows_per_wave;
    p.chunks = (int)((ncand + rpc - 1) / rpc);
    p.rows_per_chunk = (int)rpc;
    p.subs = 1;                               // (one segment per wave)
    p.sub_rows = (int)rows_per_wave;
    p.row_cap = (int)cap_rows;                // a multiple of 32
    const size_t heads = (size_t)d.batch * d.n_q_heads;
    const size_t segs = (size_t)problems * p.chunks * kStreamWaves;
    const size_t entry_bytes = 4 + d.n_sub;   // header + code bytes
    p.off_thr = 0;
    p.off_route = (p.off_thr + heads * p.P0 * sizeof(int32_t) + 255) / 256 * 256;
    p.off_count = (p.off_route + heads * sizeof(uint32_t) + 255) / 256 * 256;
    p.off_cand = (p.off_count + segs * kSegMeta * sizeof(uint32_t) + 255) / 256 * 256;
    p.bytes = (p.off_cand + segs * (size_t)p.row_cap * entry_bytes + 255) / 256 * 256;
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

// Survivor entries.  The streaming pass writes, per segment (a run of rows of one wave), row_cap
// 4-byte headers followed by row_cap rows of code bytes.  A header packs the token position (20
// bits: contexts are at most 2^20 tokens) and the mask of the heads that want the row (4 bits).
template <int M>
__host__ __device__ __forceinline__ size_t segment_words(int row_cap) {
  return (size_t)row_cap * (1 + M / 4);
}
__device__ __forceinline__ uint32_t entry_pos(uint32_t w0) { return w0 & 0xfffffu; }
__device__ __forceinline__ bool entry_wanted(uint32_t w0, int r) { return (w0 >> (20 + r)) & 1u; }

// ------------------------------------------------------------------------------------------
// Exact route (also the fallback of the fast route)
// ------------------------------------------------------------------------------------------
constexpr int kKeepRows = 16;   // rows per thread the exact route keeps in registers (16384 candidates)
struct ExactLds {
  uint32_t hist[kHistBins];
  uint32_t wave_a[kExactThreads / 64];
  uint32_t wave_b[kExactThreads / 64];
  uint32_t res[2];
  // emission with resident keys: packed (above, equal) counts per round and wave, their exclusive
  // prefixes over the waves of a round, and the rounds' totals
  uint32_t round_wave[kKeepRows][kExactThreads / 64];
  uint32_t round_pre[kKeepRows][kExactThreads / 64];
  uint32_t round_tot[kKeepRows];
  // the keys of the K-th key's bin after a select level, when they are few enough to rank by counting
  uint32_t small_n;
  uint32_t small_key[kSmallList];
};

// Exact top-K for one head by the whole workgroup.  `head_table` is the head's [c][m] table in
// global memory, `meta` its four table constants, `tbl` kExactLdsBytes of LDS.  Writes
// out_idx[0..kk) ascending (and out_score); the caller has written the count and the -1 padding.
// Requires sr.kk >= 1.
template <int M>
__device__ void exact_select_block(const SeqCodes& seq_codes,
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
  // Radix digits are taken from key - key(lower bound of any score), so that the histogram bins
  // spread over the occupied range instead of all keys sharing their leading bits.
  const uint32_t k_lo = score_key(s_lo);
  // Up to kKeep rows per thread (16384 candidates: every shape that takes this route for its length)
  // are scored once and their relative keys kept in registers; the select levels and the emission
  // then work on those instead of streaming and scoring the rows again (4 passes at 4096 tokens:
  // 23 us).  Thread t owns rows lo + t + i NT, the order of the streaming loops below.
  constexpr int kKeep = kKeepRows;
  const bool resident = hi - lo <= kKeep * NT;   // (uniform)
  uint32_t keys[kKeep];
  if (resident) {
#pragma unroll
    for (int i = 0; i < kKeep; ++i) {
      const int j = lo + tid + i * NT;
      keys[i] = j < hi ? score_key(score_exact_row<M>(row_ptr<M>(seq_codes, j), tbl, sw)) - k_lo : 0u;
    }
  }
  if (sr.kk < sr.ncand) {
    int remaining = 32 - __clz(score_key(s_hi) - k_lo);   // significant bits of a relative key
    uint32_t prefix = 0, mask = 0;
#pragma unroll 1
    while (remaining > 0) {
      const int bits = remaining < 11 ? remaining : 11;
      const int shift = remaining - bits;
      const uint32_t dmask = (1u << bits) - 1u;
      for (int i = tid; i < kHistBins; i += NT) L.hist[i] = 0;
      __syncthreads();
      if (resident) {
#pragma unroll
        for (int i = 0; i < kKeep; ++i)
          if (lo + tid + i * NT < hi && (keys[i] & mask) == prefix) atomicAdd(&L.hist[(keys[i] >> shift) & dmask], 1u);
      } else {
        for (int j = lo + tid; j < hi; j += NT) {
          const uint32_t key = score_key(score_exact_row<M>(row_ptr<M>(seq_codes, j), tbl, sw)) - k_lo;
          if ((key & mask) == prefix) atomicAdd(&L.hist[(key >> shift) & dmask], 1u);
        }
      }
      __syncthreads();
      block_find_rank_desc<NT, kHistBins>([&](int i) { return L.hist[i]; }, k_rem, L.wave_a, L.res);
      const uint32_t bin = L.res[0], above = L.res[1], m_bin = L.hist[bin];
      k_rem -= above;
      prefix |= bin << shift;
      mask |= dmask << shift;
      remaining = shift;
      if (tid == 0) L.small_n = 0;
      __syncthreads();
      if (resident && remaining > 0 && m_bin <= (uint32_t)kSmallList) {   // (uniform)
        // The bin of the K-th key usually holds a handful of keys: they are listed and each member
        // counts the members above and at its own key -- the member whose range contains k_rem is the
        // K-th key.  (A crowded bin, heavy ties, goes on with the next radix level.)
#pragma unroll
        for (int i = 0; i < kKeep; ++i)
          if (lo + tid + i * NT < hi && (keys[i] & mask) == prefix) L.small_key[atomicAdd(&L.small_n, 1u)] = keys[i];
        __syncthreads();
        if ((uint32_t)tid < m_bin) {
          const uint32_t key = L.small_key[tid];
          uint32_t gt = 0, eq = 0;
          for (uint32_t u = 0; u < m_bin; ++u) {
            const uint32_t ku = L.small_key[u];
            gt += ku > key ? 1u : 0u;
            eq += ku == key ? 1u : 0u;
          }
          if (gt < k_rem && k_rem <= gt + eq) {   // every member at the K-th key writes the same two words
            L.res[0] = key;
            L.res[1] = k_rem - gt;
          }
        }
        __syncthreads();
        prefix = L.res[0];
        k_rem = L.res[1];
        remaining = 0;
        __syncthreads();   // L.res is rewritten by the caller's next use
      }
    }
    kth = prefix + k_lo;
  }

  // Ordered emission: keys above the K-th, plus the first k_rem positions that equal it.
  uint32_t eq_seen = 0, out_n = 0;
  const bool take_all = sr.kk >= sr.ncand;
  auto emit_round = [&](int base, bool have_key, uint32_t rel_key, bool& done) {
    const int j = base + tid;
    int32_t s = 0;
    uint32_t gt = 0, eq = 0;
    if (j < hi) {
      s = have_key ? key_score(rel_key + k_lo) : score_exact_row<M>(row_ptr<M>(seq_codes, j), tbl, sw);
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
    done = out_n >= (uint32_t)sr.kk;   // (uniform)
  };
  bool done = false;
  if (resident) {
    // All rounds at once: a wave scan of the packed (above, equal) flags per round, one scan over the
    // waves of every round (16 lanes per round), then each thread places its winners -- two barriers
    // instead of four per round.  A winner's slot is the number of keys above the K-th before it plus
    // the number of equal keys before it that still fit (both counts grow with the position).
    constexpr int NW = NT / 64;
    static_assert(kKeep * NW <= NT && NW == 16, "one lane per (round, wave), 16 waves per round");
    const int lane = tid & 63, wave = tid >> 6;
    uint32_t flags = 0;        // bit 2 i: above the K-th key, bit 2 i + 1: equal to it
    uint32_t pre[kKeep];
#pragma unroll
    for (int i = 0; i < kKeep; ++i) {
      uint32_t own = 0;
      if (lo + tid + i * NT < hi) {
        const uint32_t key = keys[i] + k_lo;
        own = take_all ? 1u : (key > kth ? 1u : (key == kth ? 0x10000u : 0u));
      }
      flags |= ((own & 1u) | ((own >> 16) << 1)) << (2 * i);
      const uint32_t v = wave_inclusive_scan(own);
      pre[i] = v - own;
      if (lane == 63) L.round_wave[i][wave] = v;
    }
    __syncthreads();
    if (tid < kKeep * NW) {
      const int i = tid / NW, w = tid % NW;
      const uint32_t own = L.round_wave[i][w];
      uint32_t v = own;
#pragma unroll
      for (int off = 1; off < NW; off <<= 1) {
        const uint32_t n = __shfl_up(v, off, NW);
        if (w >= off) v += n;
      }
      L.round_pre[i][w] = v - own;
      if (w == NW - 1) L.round_tot[i] = v;
    }
    __syncthreads();
    uint32_t gt_base = 0, eq_base = 0;
#pragma unroll
    for (int i = 0; i < kKeep; ++i) {
      const uint32_t f = (flags >> (2 * i)) & 3u;
      if (f) {
        const uint32_t p = pre[i] + L.round_pre[i][wave];
        const uint32_t gt_before = gt_base + (p & 0xffffu), eq_before = eq_base + (p >> 16);
        if ((f & 1u) || eq_before < k_rem) {
          const uint32_t slot = gt_before + min(eq_before, k_rem);
          out_idx[slot] = lo + tid + i * NT;
          if (out_score) out_score[slot] = (float)key_score(keys[i] + k_lo) * scale;
        }
      }
      const uint32_t tot = L.round_tot[i];
      gt_base += tot & 0xffffu;
      eq_base += tot >> 16;
    }
  } else {
#pragma unroll 1
    for (int base = lo; base < hi && !done; base += NT) emit_round(base, false, 0u, done);
  }
}

template <int M>
__global__ __launch_bounds__(kExactThreads) void select_exact_kernel(
    const uint8_t* __restrict__ codes, const int32_t* __restrict__ lut,
    const float* __restrict__ lut_scale, const int32_t* __restrict__ seq_lens,
    int32_t* __restrict__ topk_idx, int32_t* __restrict__ topk_count,
    float* __restrict__ topk_score, CodePages pg, int B, int Hq, int Hkv, int ctx_len, int64_t ctx_stride,
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
  exact_select_block<M>(seq_codes_of<M>(codes, pg, b, kv, Hkv, ctx_stride),
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
    float* __restrict__ scores_out, CodePages pg, int B, int Hq, int Hkv, int ctx_len, int64_t ctx_stride) {
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
  const SeqCodes seq_codes = seq_codes_of<M>(codes, pg, b, kv, Hkv, ctx_stride);
  const float sc = lut_scale[bh];
  for (int j = blockIdx.x * kStreamThreads + threadIdx.x; j < n; j += gridDim.x * kStreamThreads)
    scores_out[(size_t)bh * ctx_stride + j] = (float)score_exact_row<M>(row_ptr<M>(seq_codes, j), tbl, sw) * sc;
}

// ------------------------------------------------------------------------------------------
// Fast route, stage 1: sampled coarse thresholds
// ------------------------------------------------------------------------------------------
template <int M>
__global__ __launch_bounds__(kSampleThreads) void sample_threshold_kernel(
    const uint8_t* __restrict__ codes, const int32_t* __restrict__ lut,
    const int32_t* __restrict__ seq_lens, int32_t* __restrict__ thr, CodePages pg, int B, int Hq, int Hkv,
    int NG, int P0, int sample_rows, int problems, int ctx_len, int64_t ctx_stride, int top_k, int window,
    int n_sink) {
  extern __shared__ __align__(16) unsigned char dyn_lds[];
  int p, prob;
  xcd_map_sets(blockIdx.x, P0, problems, NG, prob, p);
  sample_threshold_body<M, kSampleThreads, false>(prob, p, codes, pg, lut, seq_lens, thr, B, Hq, Hkv, NG, P0, sample_rows,
                                                  ctx_len, ctx_stride, top_k, window, n_sink, dyn_lds);
}

// ------------------------------------------------------------------------------------------
// Fast route, stage 2: one pass over the code matrix
// ------------------------------------------------------------------------------------------
// RESHARED: the rows are read by more than one problem (the head groups of a KV head, placed next
// to each other on one XCD): ordinary loads, so that the line stays in that L2 for the neighbour;
// otherwise non-temporal loads (each row is read once).
// PAGED: the code rows live in a pool of pages; the page numbers of the workgroup's chunk are
// staged in LDS behind the table (up to kPageSlice of them, else they are read from the page table
// row by row), and rows are read with ordinary loads.
constexpr int kPageSlice = 2048;
template <int M, bool RESHARED, bool PAGED>
__device__ __forceinline__ void stream_select_body(
    const uint8_t* __restrict__ codes, const int32_t* __restrict__ lut,
    const int32_t* __restrict__ seq_lens, const int32_t* __restrict__ thr,
    uint32_t* __restrict__ seg_meta, uint32_t* __restrict__ cand, GridMap gm, CodePages pg, int B, int Hq, int Hkv, int G,
    int NG, int P0, int n_chunks, int rows_per_chunk, int row_cap, int ctx_len,
    int64_t ctx_stride, int top_k, int window, int n_sink) {
  constexpr int NT = kStreamThreads;
  extern __shared__ __align__(16) unsigned char dyn_lds[];
  unsigned char* tbl = dyn_lds;

  int chunk, prob, b, kv, g4;
  map_block(blockIdx.x, gm, prob, chunk);
  split_problem(prob, gm, b, kv, g4);
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const SeqRange sr = seq_range(ctx_len, seq_lens, b, window, n_sink, top_k);
  const long begin = (long)sr.sink_end + (long)chunk * rows_per_chunk;
  const int end = (int)min((long)sr.win_start, begin + rows_per_chunk);
  // A wave owns a contiguous run of rows, so its survivors come out in ascending position and
  // the segments of a problem, taken in (chunk, wave) order, are sorted by position.
  const int rows_per_wave = rows_per_chunk / kStreamWaves;
  const long wbegin = begin + (long)wv * rows_per_wave;
  const int wend = (int)min((long)end, wbegin + rows_per_wave);

  // Every (problem, chunk, wave) owns one survivor segment in HBM: no atomics, no contention.
  const size_t seg = ((size_t)prob * n_chunks + chunk) * kStreamWaves + wv;
  uint32_t* my_meta = seg_meta + seg * kSegMeta;
  // thresholds of the group's heads: requested here, combined after the table copy has been issued
  const int32_t thr_lane = request_thresholds<4>(thr, (size_t)b * Hq + kv * G + g4 * kHeadsPerGroup,
                                                G - g4 * kHeadsPerGroup, P0);
  int32_t T[4];   // padded heads never want a row
  // The scoring loop addresses the table by absolute LDS address (it must start at 0, which holds
  // because this kernel has no static LDS).  Should a toolchain ever place it elsewhere, publish
  // an overflowing segment instead: the final kernel then takes the exact route.
  const bool misplaced = (uint32_t)(uintptr_t)tbl != 0u;
  if (begin >= sr.win_start || misplaced) {   // nothing to score in this chunk: an empty segment
    if (lane < kSegMeta) my_meta[lane] = misplaced && lane == 0 ? 0xffffffffu : 0u;
    return;
  }

  LaneSwizzle<M> sw;
  sw.init(lane);
  int n_rows = 0;                  // row entries written by this wave (wave-uniform)
  int n_head[4] = {0, 0, 0, 0};    // of which wanted by each head
  // A segment is row_cap 4-byte entry headers followed by row_cap rows of code bytes.
  uint32_t* my_seg = cand + seg * segment_words<M>(row_cap);
  uint32_t* my_hdr = my_seg;
  uint4* my_codes = (uint4*)(my_seg + (size_t)row_cap);

  const bool has_rows = wbegin < wend;   // wave-uniform
  {
    const SeqCodes seq_codes = seq_codes_of<M>(codes, pg, b, kv, Hkv, ctx_stride);
    int32_t* pg_lds = (int32_t*)(dyn_lds + kCoarseLdsBytes);
    const int pg0 = PAGED ? (int)((uint32_t)begin >> seq_codes.shift) : 0;                  // first page slot of the chunk
    const int n_pg = PAGED ? (int)((uint32_t)(end - 1) >> seq_codes.shift) - pg0 + 1 : 0;   // (begin < end here)
    const bool pg_staged = PAGED && n_pg <= kPageSlice;
    // Rows are read U at a time per lane, one full step ahead of their use (two register sets
    // used alternately); loads are unconditional (row index clamped into the wave's range) so
    // that the wait before the gathers only covers the older of the two sets in flight.
    constexpr int U = 4;
    constexpr int STEP = 64 * U;
    uint4 rows_a[U][M / 16], rows_b[U][M / 16];
    auto load_rows = [&](int base, uint4 (&dst)[U][M / 16], bool pages_in_lds) {
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int j = base + u * 64 + lane;
        const int jl = j < wend ? j : wend - 1;
        const uint8_t* row;
        if (PAGED) {
          const int slot = (int)((uint32_t)jl >> seq_codes.shift);
          row = row_in_page<M>(seq_codes, pages_in_lds ? pg_lds[slot - pg0] : seq_codes.pages[slot], jl);
        } else {
          row = seq_codes.base + (size_t)jl * M;
        }
#pragma unroll
        for (int qd = 0; qd < M / 16; ++qd)
          dst[u][qd] = (RESHARED || PAGED) ? *(const uint4*)(row + ((uint32_t)(qd * 16) ^ sw.row_swz))
                                           : load_stream_u4(row + ((uint32_t)(qd * 16) ^ sw.row_swz));
      }
    };
    auto process = [&](int base, const uint4 (&rows)[U][M / 16]) {
      // Scores and the per-head "reaches the threshold" wave masks are formed together, so the
      // gathered table entries die inside this straight-line block.  The masks live in scalar
      // registers; their popcounts cost no vector instructions.
      uint64_t hit[U][4];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        uint32_t a01, a23;
        score_coarse<M, true>(rows[u], tbl, sw, a01, a23);
        const uint64_t valid = __builtin_amdgcn_ballot_w64(base + u * 64 + lane < wend);
        hit[u][0] = __builtin_amdgcn_ballot_w64((int32_t)(a01 & 0xffffu) >= T[0]) & valid;
        hit[u][1] = __builtin_amdgcn_ballot_w64((int32_t)(a01 >> 16) >= T[1]) & valid;
        hit[u][2] = __builtin_amdgcn_ballot_w64((int32_t)(a23 & 0xffffu) >= T[2]) & valid;
        hit[u][3] = __builtin_amdgcn_ballot_w64((int32_t)(a23 >> 16) >= T[3]) & valid;
        if (u & 1) __builtin_amdgcn_sched_barrier(0);   // two rows' gathers at a time: bounds live registers
      }
      // A surviving row is written once, with the mask of the heads that want it; entries keep
      // the order of the rows, so the final kernel finds a row's place among the rows a head
      // wants by counting mask bits.
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const uint64_t any = hit[u][0] | hit[u][1] | hit[u][2] | hit[u][3];
        if (any) {
          if (__builtin_amdgcn_inverse_ballot_w64(any)) {
            const int slot = (int)__builtin_amdgcn_mbcnt_hi(
                (uint32_t)(any >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)any, (uint32_t)n_rows));
            if (slot < row_cap) {   // rows past the capacity are dropped but still counted
              uint32_t hdr = (uint32_t)(base + u * 64 + lane);
#pragma unroll
              for (int r = 0; r < 4; ++r)
                hdr |= __builtin_amdgcn_inverse_ballot_w64(hit[u][r]) ? (1u << (20 + r)) : 0u;
              my_hdr[slot] = hdr;
#pragma unroll
              for (int qd = 0; qd < M / 16; ++qd)   // (row_swz: which half of the row this register holds)
                my_codes[slot * (M / 16) + (qd ^ (int)(sw.row_swz >> 4))] = rows[u][qd];
            }
          }
          n_rows += __popcll(any);
#pragma unroll
          for (int r = 0; r < 4; ++r) n_head[r] += __popcll(hit[u][r]);
        }
      }
    };
    // The first rows are requested before the table is copied to LDS, so both latencies overlap.
    // (Every wave of the workgroup reaches the barrier, also one whose row range is empty.)
    if (has_rows) load_rows((int)wbegin, rows_a, false);
    load_coarse_table<M, NT>(lut, lut_layout(B, Hq, Hkv, M), prob, tbl);
    if (pg_staged)
      for (int i = tid; i < n_pg; i += NT) pg_lds[i] = seq_codes.pages[pg0 + i];
    combine_thresholds<4>(thr_lane, G - g4 * kHeadsPerGroup, P0, T);
    __syncthreads();
#pragma unroll 1
    for (int base = (int)wbegin; base < wend; base += 2 * STEP) {
      load_rows(base + STEP, rows_b, pg_staged);
      process(base, rows_a);
      load_rows(base + 2 * STEP, rows_a, pg_staged);
      process(base + STEP, rows_b);
    }
  }
  // header of the segment: rows written, rows per head
  if (lane < kSegMeta) {
    uint32_t v = 0;
    if (lane == 0) v = (uint32_t)n_rows;
#pragma unroll
    for (int r = 0; r < 4; ++r)
      if (lane == 1 + r) v = (uint32_t)n_head[r];
    my_meta[lane] = v;
  }
}

#define A2ATS_STREAM_ARGS                                                                          \
  const uint8_t *__restrict__ codes, const int32_t *__restrict__ lut,                             \
      const int32_t *__restrict__ seq_lens, const int32_t *__restrict__ thr,                      \
      uint32_t *__restrict__ seg_meta, uint32_t *__restrict__ cand, GridMap gm, CodePages pg,      \
      int B, int Hq, int Hkv, int G, int NG, int P0, int n_chunks, int rows_per_chunk,             \
      int row_cap, int ctx_len, int64_t ctx_stride, int top_k, int window, int n_sink
#define A2ATS_STREAM_PASS                                                                          \
  codes, lut, seq_lens, thr, seg_meta, cand, gm, pg, B, Hq, Hkv, G, NG, P0, n_chunks,              \
      rows_per_chunk, row_cap, ctx_len, ctx_stride, top_k, window, n_sink

// 64 KB of LDS per workgroup (72 KB with a staged page slice).  M = 16: 128 VGPRs -> 4 waves per
// SIMD (two workgroups per CU).
__global__ __launch_bounds__(kStreamThreads) __attribute__((amdgpu_waves_per_eu(4, 4)))
void stream_select_kernel16(A2ATS_STREAM_ARGS) { stream_select_body<16, false, false>(A2ATS_STREAM_PASS); }
__global__ __launch_bounds__(kStreamThreads) __attribute__((amdgpu_waves_per_eu(4, 4)))
void stream_select_kernel16r(A2ATS_STREAM_ARGS) { stream_select_body<16, true, false>(A2ATS_STREAM_PASS); }
__global__ __launch_bounds__(kStreamThreads) __attribute__((amdgpu_waves_per_eu(4, 4)))
void stream_select_kernel16p(A2ATS_STREAM_ARGS) { stream_select_body<16, true, true>(A2ATS_STREAM_PASS); }
// M = 32: twice the row registers.
__global__ __launch_bounds__(kStreamThreads) __attribute__((amdgpu_waves_per_eu(2, 4)))
void stream_select_kernel32(A2ATS_STREAM_ARGS) { stream_select_body<32, false, false>(A2ATS_STREAM_PASS); }
__global__ __launch_bounds__(kStreamThreads) __attribute__((amdgpu_waves_per_eu(2, 4)))
void stream_select_kernel32r(A2ATS_STREAM_ARGS) { stream_select_body<32, true, false>(A2ATS_STREAM_PASS); }
__global__ __launch_bounds__(kStreamThreads) __attribute__((amdgpu_waves_per_eu(2, 4)))
void stream_select_kernel32p(A2ATS_STREAM_ARGS) { stream_select_body<32, true, true>(A2ATS_STREAM_PASS); }

// ------------------------------------------------------------------------------------------
// Fast route, stage 3: exact scores of the survivors, exact selection, ordered output
// ------------------------------------------------------------------------------------------
template <int M>
__global__ __launch_bounds__(kExactThreads) void final_select_kernel(
    const uint8_t* __restrict__ codes, const int32_t* __restrict__ lut,
    const float* __restrict__ lut_scale, const int32_t* __restrict__ seq_lens,
    const int32_t* __restrict__ thr, const uint32_t* __restrict__ seg_meta,
    const uint32_t* __restrict__ cand, uint32_t* __restrict__ route, int32_t* __restrict__ topk_idx,
    int32_t* __restrict__ topk_count, float* __restrict__ topk_score, GridMap gm, CodePages pg, int B,
    int Hq, int Hkv, int G, int NG, int P0, int n_seg, int row_cap, int cap, int ctx_len, int64_t ctx_stride,
    int top_k, int window, int n_sink) {
  constexpr int NT = kExactThreads;
  extern __shared__ __align__(16) unsigned char dyn_lds[];
  __shared__ ExactLds L;
  __shared__ uint32_t s_seg_off[513];
  __shared__ uint32_t s_overflow, s_small_n, s_kth;
  __shared__ uint32_t s_small_key[kSmallList];

  // one workgroup per (problem, head slot), on the XCD that streamed the problem
  int prob, r, b, kv, g4;
  map_block(blockIdx.x, gm, prob, r);
  split_problem(prob, gm, b, kv, g4);
  const int hg = g4 * kHeadsPerGroup + r;
  if (hg >= G) return;
  const int bh = b * Hq + kv * G + hg, tid = threadIdx.x;
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
  const SeqCodes seq_codes = seq_codes_of<M>(codes, pg, b, kv, Hkv, ctx_stride);

  // LDS carve-up: the head's exact table, survivor keys and positions
  unsigned char* tbl = dyn_lds;
  uint32_t* c_key = (uint32_t*)(dyn_lds + kExactLdsBytes);
  uint32_t* c_pos = c_key + cap;

  // Everything this workgroup needs from global memory before it can look at a survivor is
  // requested here in one go, so the latencies overlap: the segment headers, the threshold and
  // table constants of the completeness check (used at the very end), and the head's table.
  uint32_t seg_rows = 0, my_cnt = 0;
  if (tid < n_seg) {
    const uint32_t* mt = seg_meta + ((size_t)prob * n_seg + tid) * kSegMeta;
    seg_rows = mt[0];
    my_cnt = mt[1 + r];
  }
  const int32_t thr_lane = request_thresholds<1>(thr, (size_t)bh, 1, P0);
  const int32_t* meta = lut + lay.off_meta + (size_t)bh * 4;
  const int32_t m_base = meta[0], m_shift = meta[1], m_top = meta[2];
  load_exact_table<M, NT>(head_table, tbl);
  int32_t tc1[1];
  combine_thresholds<1>(thr_lane, 1, P0, tc1);
  const int32_t tc = tc1[0];
  const long proof_bound = (long)m_base + (((long)tc - 1 + M) << m_shift);
  ExactSwizzle<M> sw;
  sw.init(tid & 63);
  for (int i = tid; i < kHistBins; i += NT) L.hist[i] = 0;
  if (tid == 0) {
    s_overflow = 0;
    s_small_n = 0;
    s_kth = 0;
  }
  __syncthreads();
  // Survivor segments of this head's problem (one per chunk and wave of the streaming pass,
  // sorted by position when taken in order): exclusive prefix of the number of rows this head
  // wants in each.  n_seg <= 512 <= NT.
  __shared__ uint32_t s_seg_rows[512];
  if (tid < n_seg) {
    if (seg_rows > (uint32_t)row_cap) s_overflow = 1;
    s_seg_rows[tid] = seg_rows;
  }
  uint32_t n_c;
  const uint32_t my_off = block_exclusive_scan<NT>(my_cnt, L.wave_a, n_c);
  if (tid < n_seg) s_seg_off[tid] = my_off;
  if (tid == 0) s_seg_off[n_seg] = n_c;
  __syncthreads();
  if (s_overflow || n_c > (uint32_t)cap || n_c < (uint32_t)sr.kk) {
    if (tid == 0) route[bh] = s_overflow ? 3u : (n_c > (uint32_t)cap ? 2u : 1u);   // diagnostics only
    exact_select_block<M>(seq_codes, head_table, meta, scale, sr, oi, os, tbl, L);
    return;
  }

  // Keys are taken relative to a lower bound of every survivor's exact key (a survivor's coarse
  // score reaches the threshold, so its exact score is at least base + (Tc << s)), and the first
  // radix level spreads the 2048 bins over the range up to the largest possible score.  Both
  // bounds are known before any survivor is looked at, so the histogram is filled while the keys
  // are computed.
  const long lo_score = tc == INT32_MIN ? (long)m_base : (long)m_base + ((long)max(tc, 0) << m_shift);
  const uint32_t klo = score_key((int32_t)max(lo_score, (long)INT32_MIN + 1));
  const uint32_t khi = max(klo, score_key(m_top));
  const int nbits = 32 - __clz(khi - klo);
  const int bits1 = nbits < 11 ? nbits : 11, shift1 = nbits - bits1;
  {
    // Pass 1: pick this head's rows out of the problem's entry headers.  A group of tps lanes
    // (a power of two, at most a wave) takes a segment at a time; entries keep the order of their
    // rows, so an entry's place in the head's list is the segment's offset plus the number of
    // wanted entries before it: wave ballots restricted to the group's lanes, no exchange between
    // threads.  All header loads of a sweep are in flight together.  c_key temporarily holds where
    // the entry's code bytes are (in 16-byte units from the start of the problem's segments).
    constexpr int kInFlight = 8;
    int tps = 64;
    while (tps > 1 && tps * n_seg > NT) tps >>= 1;
    const int lane = tid & 63, gl = lane & (tps - 1);
    const uint64_t gmask = (tps == 64 ? ~0ull : ((1ull << tps) - 1ull)) << (lane - gl);
    const uint64_t gbelow = gmask & ((1ull << lane) - 1ull);
    const size_t seg_words = segment_words<M>(row_cap);
    const uint32_t* seg0 = cand + (size_t)prob * n_seg * seg_words;
    const uint32_t seg_q = (uint32_t)(seg_words / 4), codes_q = (uint32_t)row_cap / 4;   // in 16-byte units
    for (int s_ = tid / tps; s_ < n_seg; s_ += NT / tps) {
      const uint32_t n_rows = s_seg_rows[s_];
      uint32_t dst = s_seg_off[s_];   // of the next wanted entry of the group's sweep
      const uint32_t* hdr = seg0 + (size_t)s_ * seg_words;
      for (uint32_t i0 = 0; i0 < n_rows; i0 += kInFlight * tps) {   // (uniform within the group)
        // The headers are fetched together before any of them is looked at (the empty asm keeps the
        // compiler from sinking a load behind the "does this head want the row" branch, which
        // would serialise the latencies).
        uint32_t hd[kInFlight];
#pragma unroll
        for (int k = 0; k < kInFlight; ++k) hd[k] = hdr[min(i0 + k * tps + gl, n_rows - 1)];
#pragma unroll
        for (int k = 0; k < kInFlight; ++k) asm volatile("" : "+v"(hd[k]));
#pragma unroll
        for (int k = 0; k < kInFlight; ++k) {
          const uint32_t i = i0 + k * tps + gl;
          const bool want = i < n_rows && entry_wanted(hd[k], r);
          const uint64_t wm = __builtin_amdgcn_ballot_w64(want);
          const uint32_t at = dst + (uint32_t)__popcll(wm & gbelow);
          if (want && at < n_c) {   // always in range for entries the streaming pass wrote; keeps LDS writes in range whatever the workspace holds
            c_pos[at] = entry_pos(hd[k]);
            c_key[at] = (uint32_t)s_ * seg_q + codes_q + i * (M / 16);
          }
          dst += (uint32_t)__popcll(wm & gmask);
        }
      }
    }
    __syncthreads();
    // Pass 2: exact keys of this head's survivors, densely (no divergence), and their histogram.
    const uint4* codes0 = (const uint4*)seg0;
    const uint32_t last_q = (uint32_t)n_seg * seg_q - M / 16;   // the clamp below is a no-op for a consistent workspace
#pragma unroll 2
    for (uint32_t i = tid; i < n_c; i += NT) {
      const uint4* e = codes0 + min(c_key[i], last_q);
      uint4 w[M / 16];
#pragma unroll
      for (int qd = 0; qd < M / 16; ++qd) w[qd] = e[qd];
      const uint32_t key = max(score_key(score_exact<M>(w, tbl, sw)), klo) - klo;
      c_key[i] = key;
      atomicAdd(&L.hist[min(key >> shift1, (uint32_t)kHistBins - 1)], 1u);
    }
  }
  const uint32_t kmin = klo;
  __syncthreads();
  block_find_rank_desc<NT, kHistBins>([&](int i) { return L.hist[i]; }, (uint32_t)sr.kk, L.wave_a, L.res);
  const uint32_t bin1 = L.res[0], above1 = L.res[1], m_bin = L.hist[bin1];
  uint32_t k_rem = (uint32_t)sr.kk - above1;   // winners still to pick inside bin1
  uint32_t kth;                                // K-th largest relative key
  if (m_bin <= (uint32_t)kSmallList) {
    // Usual case: the bin of the K-th key holds a handful of survivors; the k_rem-th largest of
    // them is found by counting, for each member, the members above it.
    for (uint32_t i = tid; i < n_c; i += NT)
      if ((c_key[i] >> shift1) == bin1) s_small_key[atomicAdd(&s_small_n, 1u)] = c_key[i];
    __syncthreads();
    if ((uint32_t)tid < m_bin) {
      const uint32_t key = s_small_key[tid];
      uint32_t gt = 0, eq = 0;
      for (uint32_t u = 0; u < m_bin; ++u) {
        const uint32_t ku = s_small_key[u];
        gt += ku > key ? 1u : 0u;
        eq += ku == key ? 1u : 0u;
      }
      if (gt < k_rem && k_rem <= gt + eq) s_kth = key;   // every thread that qualifies holds this key
    }
    __syncthreads();
    kth = s_kth;
  } else {
    // Heavy ties: finish the radix select level by level.
    uint32_t prefix = bin1 << shift1, mask = ((1u << bits1) - 1u) << shift1;
    int remaining = shift1;
    __syncthreads();
#pragma unroll 1
    while (remaining > 0) {
      const int bits = remaining < 11 ? remaining : 11;
      const int shift = remaining - bits;
      const uint32_t dmask = (1u << bits) - 1u;
      for (int i = tid; i < kHistBins; i += NT) L.hist[i] = 0;
      __syncthreads();
      for (uint32_t i = tid; i < n_c; i += NT) {
        const uint32_t key = c_key[i];
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
    kth = prefix;
  }

  // Completeness: a row that is not a survivor has coarse score <= Tc - 1, hence exact score
  // below base + ((Tc - 1 + M) << shift).  If the K-th survivor key reaches that bound, no such
  // row can displace (or tie with) a winner.  Otherwise redo this head by the exact route.
  {
    const long kth_score = (long)key_score(kth + kmin);
    if (tc != INT32_MIN && kth_score < proof_bound) {
      if (tid == 0) route[bh] = 4u;
      exact_select_block<M>(seq_codes, head_table, meta, scale, sr, oi, os, tbl, L);
      return;
    }
    if (tid == 0) route[bh] = 0u;
  }

  // Winners: keys above the K-th, plus the first (K - #above) survivors equal to it.  Survivors
  // are in ascending position, so a winner's output slot is the number of winners before it:
  // one block scan over (above, equal) counts packed in a word.
  const uint32_t per = (n_c + NT - 1) / NT;
  const uint32_t i0 = min(n_c, (uint32_t)tid * per), i1 = min(n_c, i0 + per);
  uint32_t loc = 0;
  for (uint32_t i = i0; i < i1; ++i) {
    const uint32_t key = c_key[i];
    loc += (key > kth ? 1u : 0u) + (key == kth ? 0x10000u : 0u);
  }
  uint32_t tot;
  uint32_t pre = block_exclusive_scan<NT>(loc, L.wave_b, tot);
  const uint32_t k_eq = (uint32_t)sr.kk - (tot & 0xffffu);   // equal keys that still fit
  for (uint32_t i = i0; i < i1; ++i) {
    const uint32_t key = c_key[i];
    const uint32_t gt_before = pre & 0xffffu, eq_before = pre >> 16;
    const bool win = key > kth || (key == kth && eq_before < k_eq);
    if (win) {
      const uint32_t slot = gt_before + min(eq_before, k_eq);
      oi[slot] = (int32_t)c_pos[i];
      if (os) os[slot] = (float)key_score(key + kmin) * scale;
    }
    pre += (key > kth ? 1u : 0u) + (key == kth ? 0x10000u : 0u);
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
                     d.n_q_heads, d.n_kv_heads, plan.NG, plan.chunks * kStreamWaves);
  return hipGetLastError();
}

template <int M>
static hipError_t launch_score_topk_m(const a2ats_dims& d, const TopkPlan& plan, const uint8_t* codes,
                                      const CodePages& pg, const int32_t* lut, const float* lut_scale, int top_k, int window,
                                      int n_sink, const int32_t* seq_lens, int32_t* topk_idx,
                                      int32_t* topk_count, float* topk_score, float* scores_out,
                                      void* ws, bool presampled, hipStream_t stream, hipEvent_t ev_start,
                                      hipEvent_t ev_stop) {
  const int B = d.batch, Hq = d.n_q_heads, Hkv = d.n_kv_heads, NG = plan.NG;
  const int heads = B * Hq, problems = B * Hkv * NG;
  const size_t coarse_bytes = (size_t)kCoarseLdsBytes;
  const size_t lut1_bytes = kExactLdsBytes;
  hipError_t err;
  static LdsSlot s_dense[16], s_exact[16], s_sample[16], s_stream[16], s_stream_r[16], s_stream_p[16], s_final[16];
  if (heads == 0) return hipSuccess;

  if (scores_out) {
    if ((err = allow_dynamic_lds(score_dense_kernel<M>, lut1_bytes, s_dense)) != hipSuccess) return err;
    int gx = (d.ctx_len + kStreamThreads * 8 - 1) / (kStreamThreads * 8);
    gx = gx < 1 ? 1 : gx;
    hipLaunchKernelGGL((score_dense_kernel<M>), dim3(gx, heads), dim3(kStreamThreads), lut1_bytes, stream,
                       codes, lut, lut_scale, seq_lens, scores_out, pg, B, Hq, Hkv, d.ctx_len, d.ctx_stride);
    if ((err = hipGetLastError()) != hipSuccess) return err;
  }

  if (!plan.fast) {
    if ((err = allow_dynamic_lds(select_exact_kernel<M>, lut1_bytes, s_exact)) != hipSuccess) return err;
    hipLaunchKernelGGL((select_exact_kernel<M>), dim3(heads), dim3(kExactThreads), lut1_bytes, stream,
                       codes, lut, lut_scale, seq_lens, topk_idx, topk_count, topk_score, pg, B, Hq, Hkv,
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
                       coarse_bytes, stream, codes, lut, seq_lens, thr, pg, B, Hq, Hkv, NG, plan.P0, plan.sample_rows,
                       problems, d.ctx_len, d.ctx_stride, top_k, window, n_sink);
    if ((err = hipGetLastError()) != hipSuccess) return err;
  }

  const bool paged = pg.table != nullptr;
  auto stream_kernel = paged ? (M == 16 ? stream_select_kernel16p : stream_select_kernel32p)
                             : (M == 16 ? (NG > 1 ? stream_select_kernel16r : stream_select_kernel16)
                                        : (NG > 1 ? stream_select_kernel32r : stream_select_kernel32));
  const size_t stream_lds = coarse_bytes + (paged ? (size_t)kPageSlice * sizeof(int32_t) : 0);
  if ((err = allow_dynamic_lds(stream_kernel, stream_lds, paged ? s_stream_p : (NG > 1 ? s_stream_r : s_stream))) !=
      hipSuccess)
    return err;
  // (the index arithmetic of a workgroup -- which problem, which part of it -- is prepared here:
  // its divisions would otherwise be the first thing every wave does)
  const int G = Hq / Hkv;
  const GridMap gm_stream = make_grid_map(plan.chunks, problems, NG, Hkv);
  if (ev_start && ev_stop) {
    // events attached to the dispatch itself: their difference is the kernel's own duration
    hipExtLaunchKernelGGL(stream_kernel, dim3(plan.chunks * problems), dim3(kStreamThreads), stream_lds,
                          stream, ev_start, ev_stop, 0, codes, lut, seq_lens, thr, seg_meta, cand, gm_stream, pg, B,
                          Hq, Hkv, G, NG, plan.P0, plan.chunks, plan.rows_per_chunk,
                          plan.row_cap, d.ctx_len, d.ctx_stride, top_k, window, n_sink);
  } else {
    hipLaunchKernelGGL(stream_kernel, dim3(plan.chunks * problems), dim3(kStreamThreads), stream_lds,
                       stream, codes, lut, seq_lens, thr, seg_meta, cand, gm_stream, pg, B, Hq, Hkv, G, NG, plan.P0,
                       plan.chunks, plan.rows_per_chunk, plan.row_cap,
                       d.ctx_len, d.ctx_stride, top_k, window, n_sink);
  }
  if ((err = hipGetLastError()) != hipSuccess) return err;

  const size_t final_lds = lut1_bytes + (size_t)plan.cap * 8;
  if ((err = allow_dynamic_lds(final_select_kernel<M>, final_lds, s_final)) != hipSuccess) return err;
  hipLaunchKernelGGL((final_select_kernel<M>), dim3(problems * kHeadsPerGroup), dim3(kExactThreads),
                     final_lds, stream, codes, lut, lut_scale, seq_lens, thr, seg_meta, cand, route, topk_idx,
                     topk_count, topk_score, make_grid_map(kHeadsPerGroup, problems, NG, Hkv), pg, B, Hq, Hkv, G, NG,
                     plan.P0, plan.chunks * kStreamWaves, plan.row_cap, plan.cap, d.ctx_len, d.ctx_stride,
                     top_k, window, n_sink);
  return hipGetLastError();
}

__global__ void codes_to_pages_kernel(const uint8_t* __restrict__ rows, uint8_t* __restrict__ pool, CodePages pg,
                                      int Hkv, int n_new, int pos0, int row_bytes, int total) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;   // one 4-byte word of one row
  const int wpr = row_bytes / 4;
  if (i >= total) return;
  const int w = i % wpr, r = i / wpr, t = r % n_new, bkv = r / n_new, kv = bkv % Hkv, b = bkv / Hkv;
  const int j = pos0 + t;
  const size_t page = (size_t)pg.table[(size_t)b * pg.pages_per_seq + (j >> pg.shift)];
  const size_t dst = ((page * Hkv + kv) << pg.shift) + (size_t)(j & ((1 << pg.shift) - 1));
  ((uint32_t*)(pool + dst * row_bytes))[w] = ((const uint32_t*)(rows + (size_t)r * row_bytes))[w];
}

hipError_t launch_codes_to_pages(const a2ats_dims& d, const uint8_t* rows, int n_new, int pos0, int row_bytes,
                                 uint8_t* pool, const CodePages& pg, hipStream_t stream) {
  const long total = (long)d.batch * d.n_kv_heads * n_new * (row_bytes / 4);
  if (total == 0) return hipSuccess;
  hipLaunchKernelGGL(codes_to_pages_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream, rows, pool,
                     pg, d.n_kv_heads, n_new, pos0, row_bytes, (int)total);
  return hipGetLastError();
}

hipError_t launch_score_topk(const a2ats_dims& d, const uint8_t* codes, const CodePages& pg, const int32_t* lut,
                             const float* lut_scale, int top_k, int window, int n_sink,
                             const int32_t* seq_lens, int32_t* topk_idx, int32_t* topk_count,
                             float* topk_score, float* scores_out, void* ws, bool presampled,
                             hipStream_t stream, hipEvent_t ev_start, hipEvent_t ev_stop) {
  const TopkPlan plan = make_topk_plan(d, top_k, window, n_sink);
  if (d.n_sub == 16)
    return launch_score_topk_m<16>(d, plan, codes, pg, lut, lut_scale, top_k, window, n_sink, seq_lens,
                                   topk_idx, topk_count, topk_score, scores_out, ws, presampled, stream,
                                   ev_start, ev_stop);
  return launch_score_topk_m<32>(d, plan, codes, pg, lut, lut_scale, top_k, window, n_sink, seq_lens,
                                 topk_idx, topk_count, topk_score, scores_out, ws, presampled, stream,
                                 ev_start, ev_stop);
}

}  // namespace a2ats
